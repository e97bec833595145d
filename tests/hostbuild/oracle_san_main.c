/*
 * A main() around oracle/ag_oracle.c for the sanitizer run of tests/test_host_sanitizers.py.  TEST
 * INFRASTRUCTURE ONLY.  Reads one case (header of int32, scale, then for the fill batch and the chunk batch:
 * block tables, prefix lengths, new lengths, offsets, K_new, V_new, Q; then a list of rows), holds every array
 * in a heap block of its exact size, runs append (fill, chunk) on NaN-filled pools, attention on every row of
 * the chunk and on the listed rows, and writes the pools and both results to the output file.  There is no
 * arithmetic here: the values are compared, by the test, with the ordinary build of the same source.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    void *k_pool, *v_pool;
    int32_t num_pages, page_size, num_kv_heads, head_dim;
    int32_t dtype;
} ago_cache;

int ago_kv_append(const ago_cache *c, const void *k_new, const void *v_new, const int32_t *block_tables, int32_t max_pages,
                  const int32_t *prefix_lens, const int32_t *new_lens, const int32_t *cu_new, int32_t batch);
int ago_attn_rows(const ago_cache *c, const void *q, const int32_t *block_tables, int32_t max_pages,
                  const int32_t *prefix_lens, const int32_t *new_lens, const int32_t *cu_new, int32_t batch,
                  int32_t num_q_heads, double scale, const int32_t *row_session, const int32_t *row_index, int64_t n_rows,
                  double *out);
int ago_attn(const ago_cache *c, const void *q, const int32_t *block_tables, int32_t max_pages,
             const int32_t *prefix_lens, const int32_t *new_lens, const int32_t *cu_new, int32_t batch,
             int32_t num_q_heads, double scale, double *out);

static void *read_block(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short read\n"); exit(2); }
    return p;
}

typedef struct { int32_t *bt, *prefix, *new_lens, *cu; void *k, *v, *q; } batch_t;

static batch_t read_batch(FILE *f, int batch, int max_pages, int total, int hkv, int hq, int d, size_t es)
{
    batch_t b;
    b.bt = read_block(f, sizeof(int32_t) * (size_t)batch * max_pages);
    b.prefix = read_block(f, sizeof(int32_t) * (size_t)batch);
    b.new_lens = read_block(f, sizeof(int32_t) * (size_t)batch);
    b.cu = read_block(f, sizeof(int32_t) * (size_t)(batch + 1));
    b.k = read_block(f, es * (size_t)total * hkv * d);
    b.v = read_block(f, es * (size_t)total * hkv * d);
    b.q = read_block(f, es * (size_t)total * hq * d);
    return b;
}

static void free_batch(batch_t *b) { free(b->bt); free(b->prefix); free(b->new_lens); free(b->cu); free(b->k); free(b->v); free(b->q); }

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t h[11];
    double scale;
    if (fread(h, sizeof(int32_t), 11, f) != 11 || fread(&scale, sizeof(double), 1, f) != 1) return 2;
    const int dtype = h[0], num_pages = h[1], ps = h[2], hkv = h[3], d = h[4], hq = h[5], batch = h[6], max_pages = h[7];
    const int t_fill = h[8], t_chunk = h[9], n_rows = h[10];
    const size_t es = dtype == 0 ? 4 : 2;
    batch_t fill = read_batch(f, batch, max_pages, t_fill, hkv, hq, d, es);
    batch_t chunk = read_batch(f, batch, max_pages, t_chunk, hkv, hq, d, es);
    int32_t *rs = read_block(f, sizeof(int32_t) * (size_t)n_rows);
    int32_t *ri = read_block(f, sizeof(int32_t) * (size_t)n_rows);
    fclose(f);

    const size_t pool_bytes = es * (size_t)num_pages * hkv * ps * d;
    ago_cache c = {malloc(pool_bytes), malloc(pool_bytes), num_pages, ps, hkv, d, dtype};
    if (!c.k_pool || !c.v_pool) return 2;
    if (dtype == 0) {                                   /* poisoned like the tests' pools: quiet NaN 0x7FC00000 / 0x7FC0 */
        for (size_t i = 0; i < pool_bytes / 4; ++i) { ((uint32_t *)c.k_pool)[i] = 0x7FC00000u; ((uint32_t *)c.v_pool)[i] = 0x7FC00000u; }
    } else {
        for (size_t i = 0; i < pool_bytes / 2; ++i) { ((uint16_t *)c.k_pool)[i] = 0x7FC0u; ((uint16_t *)c.v_pool)[i] = 0x7FC0u; }
    }
    int rc = ago_kv_append(&c, fill.k, fill.v, fill.bt, max_pages, fill.prefix, fill.new_lens, fill.cu, batch);
    if (!rc) rc = ago_kv_append(&c, chunk.k, chunk.v, chunk.bt, max_pages, chunk.prefix, chunk.new_lens, chunk.cu, batch);
    const size_t full_n = (size_t)t_chunk * hq * d, some_n = (size_t)n_rows * hq * d;
    double *full = malloc(sizeof(double) * (full_n ? full_n : 1)), *some = malloc(sizeof(double) * (some_n ? some_n : 1));
    if (!full || !some) return 2;
    if (!rc) rc = ago_attn(&c, chunk.q, chunk.bt, max_pages, chunk.prefix, chunk.new_lens, chunk.cu, batch, hq, scale, full);
    if (!rc) rc = ago_attn_rows(&c, chunk.q, chunk.bt, max_pages, chunk.prefix, chunk.new_lens, chunk.cu, batch, hq, scale, rs, ri,
                                n_rows, some);
    if (rc) { fprintf(stderr, "oracle returned %d\n", rc); return 1; }
    FILE *o = fopen(argv[2], "wb");
    if (!o) return 2;
    fwrite(c.k_pool, 1, pool_bytes, o);
    fwrite(c.v_pool, 1, pool_bytes, o);
    fwrite(full, sizeof(double), full_n, o);
    fwrite(some, sizeof(double), some_n, o);
    fclose(o);
    free(full); free(some); free(c.k_pool); free(c.v_pool); free(rs); free(ri);
    free_batch(&fill);
    free_batch(&chunk);
    return 0;
}
