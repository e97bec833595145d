/*
 * CPU oracle for paged-KV softmax attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  It shares no code with the GPU path and must never be called from
 * it: only the tests, the smoke check and the benchmark's cpu_baseline leg
 * load it.
 *
 * What it computes.  The paper splits serving work into three request classes
 * (Sec. I; Sec. II-A; Fig. 1): a cold prefill runs full causal attention over
 * a whole prompt and builds the KV cache; a resume prefill appends a chunk to
 * a cached context; a decode step produces one token per session from the
 * cached keys and values.  The paper never writes the attention formula down
 * (it says "full attention" and reuses an existing engine's kernels), so the
 * reading taken here is the textbook one: scaled dot-product softmax.
 * All three classes are one rule with different (prefix, new) lengths:
 *
 *   session s has P_s cached tokens and N_s new ones; new row i sits at
 *   logical position pos = P_s + i and sees keys j = 0 .. pos, whatever class
 *   it belongs to (cold: P_s = 0; resume: P_s > 0; decode: N_s = 1 and the
 *   step's own key/value are already appended, so pos = ctx_len - 1).
 *
 *     x_j = scale * sum_d Q[s,i,h,d] * K(s,g,j)[d]          g = h / G
 *     m   = max_j x_j,   w_j = exp(x_j - m),   Z = sum_j w_j
 *     O[s,i,h,:] = ( sum_j w_j * V(s,g,j)[:] ) / Z
 *
 * K(s,g,j) and V(s,g,j) are always fetched through the session's block
 * table: page = bt[s][j / page_size], slot = j % page_size, pool layout
 * [page][kv_head][slot][d].  Query head h reads KV head h / G with
 * G = Hq / Hkv (contiguous groups).  Subtracting m changes nothing
 * mathematically (softmax is shift invariant) and keeps exp() in range.
 *
 * Precision: every stored input (fp32, or bf16 as raw 16-bit patterns) is
 * widened exactly to double; all arithmetic is double; nothing is rounded.
 * There is no blocking, no fusion and no reordering: keys are visited in
 * logical order 0..pos, twice (scores, then the weighted sum).
 *
 * Pins (tests/test_oracle_*.py, all CPU): dense brute force on tiny inputs
 * written independently in NumPy; closed forms (constant keys -> running mean
 * of V, one key -> v_0, two keys -> logistic mix); invariants (convexity,
 * linearity in V, key-shift and key-permutation invariance); the equalities
 * the three classes imply (resume == tail rows of a cold prefill of the
 * concatenation, decode == last row of a prefill); a dictionary model of the
 * append index map; page-permutation invariance.
 * The paper prints no numeric value for this path, so parity with the paper's
 * own numbers is unpinned; every pin above is mathematical.
 *
 * The OpenMP pragma only spreads independent output rows over host threads;
 * each row's arithmetic is the sequential loop below.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { AGO_F32 = 0, AGO_BF16 = 1 };

enum {
    AGO_OK = 0,
    AGO_BAD_ARG = -1,
    AGO_BAD_PAGE = -2,   /* a block-table entry outside [0, num_pages) was needed */
    AGO_NO_MEM = -3
};

typedef struct {
    void *k_pool, *v_pool;          /* [num_pages][num_kv_heads][page_size][head_dim] */
    int32_t num_pages, page_size, num_kv_heads, head_dim;
    int32_t dtype;                  /* AGO_F32 or AGO_BF16 */
} ago_cache;

static size_t elem_size(int dtype) { return dtype == AGO_F32 ? 4u : 2u; }

/* exact widening of one stored element */
static double load_elem(const void *base, size_t idx, int dtype)
{
    if (dtype == AGO_F32)
        return (double)((const float *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* element offset of (page, kv_head, slot, 0) in a pool */
static size_t pool_offset(const ago_cache *c, int64_t page, int g, int slot)
{
    return (((size_t)page * c->num_kv_heads + g) * c->page_size + slot) * (size_t)c->head_dim;
}

static int check_cache(const ago_cache *c)
{
    if (!c || !c->k_pool || !c->v_pool) return AGO_BAD_ARG;
    if (c->num_pages <= 0 || c->page_size <= 0 || c->num_kv_heads <= 0 || c->head_dim <= 0) return AGO_BAD_ARG;
    if (c->dtype != AGO_F32 && c->dtype != AGO_BF16) return AGO_BAD_ARG;
    return AGO_OK;
}

int ago_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * KV append: the cache-building half of a prefill (Sec. II-A) and the one
 * token a decode step adds.  Pure index map + byte copy:
 *   token t = cu_new[s] + i of session s goes to logical position P_s + i,
 *   i.e. page bt[s][(P_s+i) / ps], slot (P_s+i) % ps, for every KV head.
 * Host pointers throughout.
 */
int ago_kv_append(const ago_cache *c, const void *k_new, const void *v_new,   /* [T][Hkv][D] */
                  const int32_t *block_tables, int32_t max_pages,
                  const int32_t *prefix_lens, const int32_t *new_lens, const int32_t *cu_new,
                  int32_t batch)
{
    int rc = check_cache(c);
    if (rc) return rc;
    if (!k_new || !v_new || !block_tables || !prefix_lens || !new_lens || !cu_new || batch < 0 || max_pages <= 0)
        return AGO_BAD_ARG;
    const size_t row = (size_t)c->head_dim * elem_size(c->dtype);
    for (int s = 0; s < batch; ++s) {
        for (int i = 0; i < new_lens[s]; ++i) {
            const int64_t pos = (int64_t)prefix_lens[s] + i;
            const int64_t lp = pos / c->page_size;
            const int slot = (int)(pos % c->page_size);
            if (lp >= max_pages) return AGO_BAD_ARG;
            const int64_t page = block_tables[(size_t)s * max_pages + lp];
            if (page < 0 || page >= c->num_pages) return AGO_BAD_PAGE;
            const size_t t = (size_t)cu_new[s] + i;
            for (int g = 0; g < c->num_kv_heads; ++g) {
                const size_t src = (t * c->num_kv_heads + g) * row;
                const size_t dst = pool_offset(c, page, g, slot) * elem_size(c->dtype);
                memcpy((char *)c->k_pool + dst, (const char *)k_new + src, row);
                memcpy((char *)c->v_pool + dst, (const char *)v_new + src, row);
            }
        }
    }
    return AGO_OK;
}

/*
 * One output row: session s, new-row i, query head h.  `x` is scratch for
 * pos+1 scores.  Writes head_dim doubles to `out`.
 */
static int attend_row(const ago_cache *c, const void *q, size_t q_row,        /* q_row: element offset of Q[t][h][0] */
                      const int32_t *bt_row, int32_t max_pages,
                      int64_t pos, int g, double scale, double *x, double *out)
{
    const int D = c->head_dim, ps = c->page_size, dt = c->dtype;
    /* scores over every visible key, in logical order */
    double m = -INFINITY;
    for (int64_t j = 0; j <= pos; ++j) {
        const int64_t lp = j / ps;
        if (lp >= max_pages) return AGO_BAD_ARG;
        const int64_t page = bt_row[lp];
        if (page < 0 || page >= c->num_pages) return AGO_BAD_PAGE;
        const size_t ko = pool_offset(c, page, g, (int)(j % ps));
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += load_elem(q, q_row + d, dt) * load_elem(c->k_pool, ko + d, dt);
        x[j] = scale * dot;
        if (x[j] > m) m = x[j];
    }
    /* softmax weights and the weighted sum of values */
    double Z = 0.0;
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    for (int64_t j = 0; j <= pos; ++j) {
        const double w = exp(x[j] - m);
        Z += w;
        const size_t vo = pool_offset(c, bt_row[j / ps], g, (int)(j % ps));
        for (int d = 0; d < D; ++d)
            out[d] += w * load_elem(c->v_pool, vo + d, dt);
    }
    for (int d = 0; d < D; ++d) out[d] /= Z;
    return AGO_OK;
}

/*
 * Attention for a chosen list of rows: rows[r] = (session, new-row index);
 * all Hq heads of each listed row are produced, out is [n_rows][Hq][D]
 * doubles.  The full result is the list of every row (ago_attn below);
 * a sampled list makes full-size workloads checkable one row at a time.
 */
int ago_attn_rows(const ago_cache *c, const void *q,                           /* [T][Hq][D] stored dtype */
                  const int32_t *block_tables, int32_t max_pages,
                  const int32_t *prefix_lens, const int32_t *new_lens, const int32_t *cu_new,
                  int32_t batch, int32_t num_q_heads, double scale,
                  const int32_t *row_session, const int32_t *row_index, int64_t n_rows,
                  double *out)
{
    int rc = check_cache(c);
    if (rc) return rc;
    if (!q || !block_tables || !prefix_lens || !new_lens || !cu_new || !out || batch < 0 || max_pages <= 0)
        return AGO_BAD_ARG;
    if (num_q_heads <= 0 || num_q_heads % c->num_kv_heads != 0) return AGO_BAD_ARG;
    if (n_rows > 0 && (!row_session || !row_index)) return AGO_BAD_ARG;
    const int G = num_q_heads / c->num_kv_heads;
    const int D = c->head_dim;

    int64_t longest = 0;
    for (int64_t r = 0; r < n_rows; ++r) {
        const int s = row_session[r], i = row_index[r];
        if (s < 0 || s >= batch || i < 0 || i >= new_lens[s] || prefix_lens[s] < 0) return AGO_BAD_ARG;
        const int64_t ctx = (int64_t)prefix_lens[s] + i + 1;
        if (ctx > longest) longest = ctx;
    }

    int status = AGO_OK;
    const int64_t n_out = n_rows * num_q_heads;
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)(longest > 0 ? longest : 1));
        if (!x) {
#pragma omp critical
            status = AGO_NO_MEM;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t o = 0; o < n_out; ++o) {
                const int64_t r = o / num_q_heads;
                const int h = (int)(o % num_q_heads);
                const int s = row_session[r], i = row_index[r];
                const size_t t = (size_t)cu_new[s] + i;
                const int err = attend_row(c, q, (t * num_q_heads + h) * (size_t)D,
                                           block_tables + (size_t)s * max_pages, max_pages,
                                           (int64_t)prefix_lens[s] + i, h / G, scale, x,
                                           out + (size_t)o * D);
                if (err) {
#pragma omp critical
                    status = err;
                }
            }
        }
        free(x);
    }
    return status;
}

/* Every new row of every session; out is [T][Hq][D] doubles, T = cu_new[batch]. */
int ago_attn(const ago_cache *c, const void *q,
             const int32_t *block_tables, int32_t max_pages,
             const int32_t *prefix_lens, const int32_t *new_lens, const int32_t *cu_new,
             int32_t batch, int32_t num_q_heads, double scale, double *out)
{
    if (!new_lens || !cu_new || batch < 0) return AGO_BAD_ARG;
    int64_t total = 0;
    for (int s = 0; s < batch; ++s) {
        if (new_lens[s] < 0 || cu_new[s] != total) return AGO_BAD_ARG;
        total += new_lens[s];
    }
    int32_t *rs = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total > 0 ? total : 1));
    int32_t *ri = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total > 0 ? total : 1));
    if (!rs || !ri) { free(rs); free(ri); return AGO_NO_MEM; }
    int64_t r = 0;
    for (int s = 0; s < batch; ++s)
        for (int i = 0; i < new_lens[s]; ++i) { rs[r] = s; ri[r] = i; ++r; }
    const int rc = ago_attn_rows(c, q, block_tables, max_pages, prefix_lens, new_lens, cu_new,
                                 batch, num_q_heads, scale, rs, ri, total, out);
    free(rs);
    free(ri);
    return rc;
}
