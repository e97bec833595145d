// One launch for the decode queue of the paper's scheduler: decodes and short resume prefills together
// (paper Sec. III-A: short resume prefills are merged with decodes to improve parallelism; Algorithm 1 admits
// a request to Q_D when it is a decode or no longer than B_prefill).  bf16, head_dim 128, page 16.
//
// A session brings N >= 0 new query rows at positions P .. P + N - 1 (a decode is N = 1) that attend causally
// to the session's keys: the semantics of the resume prefill.  The work is cut the way the decode step cuts
// it - the keys a session's rows may see are split over workgroups, partial (m, l, O) per split, merged in
// split order - because with few rows per session the launch is bound by reading K and V:
//
//   plan kernel     lists the items.  A group is tq = 16 / G consecutive rows of one session (G = query heads
//                   per KV head): its tq x G (row, head) pairs fill the 16 columns of the matrix instruction
//                   that the decode step leaves mostly empty.  Two kinds of item:
//                     keys item  up to R groups; the four waves of a workgroup split the KEYS of the part, as in
//                                the decode step, each K / V step loaded once into registers for the R groups;
//                     rows item  up to 4 R groups (32 rows at G = 4, R = 2); the four waves split the ROWS and
//                                all walk the same keys, which the workgroup brings into LDS once per step by
//                                direct global-to-LDS loads (two stages), so a session's keys are fetched once
//                                per 4 R groups instead of once per R.
//                   Sessions with at most R groups of rows (decodes among them) become one keys item; longer
//                   chunks become rows items plus, for a remainder of at most R groups, one keys item.
//   split kernel    one workgroup per (item, KV head, split of the keys the item's last row may see), with a
//                   visibility limit per column.
//   merge kernel    one workgroup per (row, head) combines the splits in split order.
//
// Items of one (session, KV head, split) are dealt to the same XCD (their linear workgroup ids differ by a
// multiple of splits * KV heads, itself a multiple of 8 at 8 KV heads), so what they fetch again comes from
// that XCD's L2.
#include <algorithm>
#include <atomic>

#include "attn_split_common.h"
#include "attn_tile32.h"
#include "lds_dma.h"

namespace ag {

namespace {

using namespace splitk;

enum { kKeysItem = 0, kRowsItem = 1 };

// plan[0] = number of items; item i is plan[4 + 4i ..]: session, first row (within the session's chunk), rows, kind.
// row_ctx[row] = keys the item that holds query row `row` was cut over: prefix + rows of the chunk up to the
// item's last (what the merge kernel needs to count the row's partials, without walking plan -> session -> prefix).
// rk: rows of a full keys item; rw: rows of a full rows item, 0 if the launch has no rows items.
__device__ __forceinline__ int items_of(int n, int rk, int rw)
{
    if (rw == 0) return (n + rk - 1) / rk;
    return n / rw + (n % rw ? 1 : 0);
}

__global__ __launch_bounds__(256) void merged_plan_kernel(const int32_t* __restrict__ new_lens,
                                                          const int32_t* __restrict__ prefix_lens,
                                                          const int32_t* __restrict__ cu_new, int batch,
                                                          int total_rows, int rk, int rw,
                                                          int32_t* __restrict__ plan,
                                                          int32_t* __restrict__ row_ctx)
{
    __shared__ int scan[256];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < batch; base += 256) {
        const int s = base + threadIdx.x;
        const int n = s < batch ? new_lens[s] : 0;
        const int P = (s < batch && prefix_lens) ? prefix_lens[s] : 0;
        const int mine = items_of(n, rk, rw);
        scan[threadIdx.x] = mine;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {   // inclusive scan
            const int v = threadIdx.x >= off ? scan[threadIdx.x - off] : 0;
            __syncthreads();
            scan[threadIdx.x] += v;
            __syncthreads();
        }
        const int first = carry + scan[threadIdx.x] - mine;
        const int step = rw ? rw : rk;
        for (int i = 0; i < mine && first + i < total_rows; ++i) {     // (lengths that contradict the host's total
            const int t0 = i * step;                                    //  never write past the plan)
            const int nt = min(step, n - t0);
            int32_t* e = plan + 4 + 4 * (first + i);
            e[0] = s; e[1] = t0; e[2] = nt;
            e[3] = (rw && nt > rk) ? kRowsItem : kKeysItem;
            const int row0 = cu_new[s] + t0;
            for (int x = 0; x < nt && row0 + x < total_rows; ++x) row_ctx[row0 + x] = P + t0 + nt;
        }
        __syncthreads();
        if (threadIdx.x == 255) carry += scan[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) plan[0] = min(carry, total_rows);
}

// A lane's 8 weights under the reference maximum may sum to this much before the ordered path takes over.
constexpr float kWeightSumLimit = 16384.0f;

constexpr int kSmemBytes = 4 * 16 * D * 4 + 2 * 4 * 16 * 4;     // 33280: partials of four waves, or two K/V stages

struct ItemCtx {        // what both kinds of item need; uniform over the workgroup
    int s, t0, nt, split, g;
    int P, ctx_all, ctx, start, part;
};

// ---- keys item: the decode step's loop with R column groups --------------------------------------------------
template <int kSteps, int R>
__device__ __forceinline__ void keys_item(const AttnArgs& a, float* __restrict__ ws_o, float* __restrict__ ws_ml,
                                          int n_splits_max, int tq, const ItemCtx& it, unsigned char* smem)
{
    float (*s_o)[16][D] = reinterpret_cast<float (*)[16][D]>(smem);                 // per wave, per column of one group
    float (*s_m)[16] = reinterpret_cast<float (*)[16]>(smem + 4 * 16 * D * 4);
    float (*s_l)[16] = s_m + 4;

    const int s = it.s, t0 = it.t0, nt = it.nt, split = it.split, g = it.g;
    const int P = it.P, ctx_all = it.ctx_all, ctx = it.ctx, start = it.start;
    const int wave_tok = it.part >> 2;

    const int hkv = a.c.hkv, hq = a.hq;
    const int G = hq / hkv;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, c = lane >> 4;
    const int wstart = start + w * wave_tok;

    const __bf16* kpool = (const __bf16*)a.c.k;
    const __bf16* vpool = (const __bf16*)a.c.v;

    // column r of group j = (row j * tq + r / G of the item, head r % G of the KV head's group); columns
    // without a row carry a zero query and the visibility of the item's last row
    const int col_row = r / G, col_head = r - col_row * G;
    int pos[R];
    bf16x8 qf[R][4];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int row = j * tq + col_row;
        const bool on = col_row < tq && row < nt;
        pos[j] = P + t0 + (on ? row : nt - 1);
        const int64_t q_row = (int64_t)a.cu_new[s] + t0 + (on ? row : 0);
        const __bf16* qrow = (const __bf16*)a.q + (q_row * hq + (int64_t)g * G + col_head) * D + c * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 x = ld16(qrow + kk * 32);
            if (!on) x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qf[j][kk] = x;
        }
    }

    const int n_pages_ctx = (ctx + PS - 1) >> 4;
    int my_pid;
    {
        const int lp = min((wstart >> 4) + (lane & (2 * kSteps - 1)), n_pages_ctx - 1);
        my_pid = a.bt[(int64_t)s * a.max_pages + lp];
    }
    const int n_steps = wstart < ctx ? min(wave_tok >> 5, (ctx - wstart + 31) >> 5) : 0;   // uniform over the wave

    const float sl2 = a.scale * kLog2e;
    float m[R], lsum[R];
    f32x4 o[R][8];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        m[j] = -INFINITY;
        lsum[j] = 0.0f;
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) o[j][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // operand addressing as in the decode step: score row r is slot (r & 7) of page (r >> 3) of the step, the
    // second score product takes slots 8..15; lane group c owns the 8 keys of value chunk (c & 1) of page (c >> 1)
    const int k_pg = r >> 3;
    const int k_off = (c * PS + (r & 7)) * 8;
    const int v_pg = c >> 1;
    const int v_off = ((c & 1) * D + r) * 8;

#pragma unroll
    for (int st = 0; st < kSteps; ++st) {
        if (st < n_steps) {
            StepRegs x;
            {
                const int64_t pA = __builtin_amdgcn_readlane(my_pid, 2 * st);
                const int64_t pB = __builtin_amdgcn_readlane(my_pid, 2 * st + 1);
                const __bf16* kp = kpool + ((k_pg ? pB : pA) * hkv + g) * (int64_t)(D * PS) + k_off;
                const __bf16* vp = vpool + ((v_pg ? pB : pA) * hkv + g) * (int64_t)(D * PS) + v_off;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    x.k1[kk] = ld16_stream(kp + kk * 4 * PS * 8);
                    x.k2[kk] = ld16_stream(kp + kk * 4 * PS * 8 + 64);
                }
#pragma unroll
                for (int mb = 0; mb < 8; ++mb) x.v[mb] = ld16_stream(vp + mb * 16 * 8);
            }
            const int tok0 = wstart + st * 32;
            const int tokb = tok0 + (c >> 1) * PS + (c & 1) * 4;
#pragma unroll
            for (int j = 0; j < R; ++j) {
                f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k1[kk], qf[j][kk], s1, 0, 0, 0);
                    s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k2[kk], qf[j][kk], s2, 0, 0, 0);
                }
                // s1[i]: key tokb + i, s2[i]: key tokb + 8 + i, of column r
                const int keep = pos[j] + 1 - tokb;  // key tokb + i is visible to this column iff i < keep
                float xs[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    xs[i] = (i < keep) ? s1[i] * sl2 : -INFINITY;
                    xs[4 + i] = (8 + i < keep) ? s2[i] * sl2 : -INFINITY;
                }
                float mx = fmaxf(fmaxf(fmaxf(xs[0], xs[1]), fmaxf(xs[2], xs[3])), fmaxf(fmaxf(xs[4], xs[5]), fmaxf(xs[6], xs[7])));
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m[j], mx);
                // a column may see none of this wave's keys so far (its row lies before them): keep the exponents finite
                const float m_ref = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f(m[j] - m_ref);
                float psum = 0.f;
                bf16x8 pb;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float p = __builtin_amdgcn_exp2f(xs[e] - m_ref);
                    psum += p;
                    pb[e] = (__bf16)p;
                }
                lsum[j] = lsum[j] * alpha + psum;
                m[j] = m_new;
                if (j == 0 && tok0 + 32 > ctx_all) {   // slots past the session's last token may hold anything, NaN included
                    const int keep_v = ctx_all - tokb;
#pragma unroll
                    for (int mb = 0; mb < 8; ++mb) x.v[mb] = keep_quads(x.v[mb], keep_v, keep_v - 8);
                }
#pragma unroll
                for (int mb = 0; mb < 8; ++mb) {
                    o[j][mb] *= alpha;
                    o[j][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.v[mb], pb, o[j][mb], 0, 0, 0);
                }
            }
        }
    }

    // the four waves' partials of one group at a time through LDS
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int rows_here = min(tq, nt - j * tq);          // rows of group j; uniform over the workgroup
        if (rows_here <= 0) break;
        float l = lsum[j];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (j > 0) __syncthreads();                          // the previous group's readers are done
        // o[j][mb][i] is O^T[d = mb*16 + c*4 + i][column r]
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) *reinterpret_cast<f32x4*>(&s_o[w][r][mb * 16 + c * 4]) = o[j][mb];
        if (c == 0) { s_m[w][r] = m[j]; s_l[w][r] = l; }
        __syncthreads();
        const int n_cols = rows_here * G;
        for (int idx = threadIdx.x; idx < n_cols * D; idx += 256) {
            const int col = idx >> 7, d = idx & (D - 1);
            float ms = s_m[0][col];
#pragma unroll
            for (int ww = 1; ww < 4; ++ww) ms = fmaxf(ms, s_m[ww][col]);
            float acc = 0.f, lt = 0.f;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                const float mw = s_m[ww][col];
                const float f = mw == -INFINITY ? 0.f : exp2f(mw - ms);    // a wave that saw no key of this column
                acc += f * s_o[ww][col][d];
                lt += f * s_l[ww][col];
            }
            const int crow = col / G, chead = col - crow * G;
            const int64_t slot = (((int64_t)a.cu_new[s] + t0 + j * tq + crow) * hq + (int64_t)g * G + chead) * n_splits_max + split;
            ws_o[slot * D + d] = acc;
            if (d == 0) { ws_ml[slot * 2] = ms; ws_ml[slot * 2 + 1] = lt; }
        }
    }
}

// ---- rows item: four waves x 32 columns over the same keys, in the prefill kernel's 64-key tiles ---------------
// Wave w holds column groups 2w and 2w + 1 of the item (group j = tokens j * tq .. + tq - 1, column r of a group =
// token r / G, head r % G): 32 columns, the B operand of the 32x32x16 products.  The part's keys are walked in
// tiles of 64 (four pages) that the workgroup brings into LDS by direct global-to-LDS loads - three K stages,
// two V stages, tile layouts and software pipeline as in the prefill kernel (attn_tile32.h) - and every wave
// writes the partial (m, l, O) of its columns for the part straight to the workspace.
constexpr int kRowsLds = (tile32::kKStages + 2) * tile32::kTile;        // 80 KiB

template <int kSteps>
__device__ __forceinline__ void rows_item(const AttnArgs& a, float* __restrict__ ws_o, float* __restrict__ ws_ml,
                                          int n_splits_max, int tq, const ItemCtx& it, unsigned char* lds)
{
    using tile32::BN;
    using tile32::kKStages;
    using tile32::kTile;
    constexpr int kPer = 4;                 // direct loads per wave for a K tile, and for a V tile
    const int s = it.s, g = it.g, P = it.P, t0 = it.t0, nt = it.nt;
    const int hkv = a.c.hkv, hq = a.hq, G = hq / hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int wu = __builtin_amdgcn_readfirstlane(w);           // the same value, known to be uniform
    const int n = lane & 31, hi = lane >> 5;

    // key tiles of the part: absolute tiles tb .. tb + n_tiles - 1 (parts start at multiples of 128 keys)
    const int end = min(it.ctx, it.start + it.part);
    const int tb = it.start / BN;
    const int n_tiles = (end - 1) / BN + 1 - tb;                 // >= 1

    // this lane's column; columns without a row carry the item's last row (their results are not stored)
    const int r = n & 15;
    const int col_row = r / G, col_head = r - col_row * G;
    const int token = (2 * w + (n >> 4)) * tq + col_row;
    const bool on = col_row < tq && token < nt;
    const int row = on ? token : nt - 1;
    const int qpos = P + t0 + row;                               // logical position of this lane's query
    const int w_first = 2 * w * tq;                              // the wave's first token
    const int w_last = min(nt, w_first + 2 * tq) - 1;            // ... and last
    // tiles of the part this wave uses (none if it has no rows, or if the part lies above all of them), and the
    // first tile holding a key its first row may not see
    const int wave_tiles = w_first < nt ? max(0, min(n_tiles, (P + t0 + w_last) / BN + 1 - tb)) : 0;
    const int first_masked = (P + t0 + w_first + 1) / BN - tb;

    const __bf16* kpool = (const __bf16*)a.c.k;
    const __bf16* vpool = (const __bf16*)a.c.v;
    // the block table is read-only for the kernel's lifetime: through the constant address space the (uniform)
    // page-id loads are scalar loads
    typedef const __attribute__((address_space(4))) int32_t* cptr_t;
    const cptr_t bt = (cptr_t)(uintptr_t)(a.bt + (int64_t)s * a.max_pages);
    const int last_page = (it.ctx_all - 1) >> 4;

    // Q^T as B operand: column n, k-step ks covers channels ks * 16 + hi * 8 .. + 7
    bf16x8 qf[8];
    {
        const __bf16* qp = (const __bf16*)a.q + (((int64_t)a.cu_new[s] + t0 + row) * hq + (int64_t)g * G + col_head) * D + hi * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = ld16(qp + ks * 16);
    }

    unsigned char* const k_lds = lds;                            // K tile t at k_lds + (t % 3) * kTile
    unsigned char* const v_lds = lds + kKStages * kTile;         // V tile t at v_lds + (t % 2) * kTile
    const int kpg = lane >> 4, kslot = lane & 15;                // K: lane = key of the tile (page, slot)
    const int kmask[4] = {kpg == 0 ? -1 : 0, kpg == 1 ? -1 : 0, kpg == 2 ? -1 : 0, kpg == 3 ? -1 : 0};
    struct Pages { int k; int v; };                              // this LANE's page of a K tile; the wave's page of a V tile
    auto pages_of = [&](int tk, int tv, Pages& pg) {             // absolute tile numbers
        int pid[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pid[i] = bt[min(tk * 4 + i, last_page)];
        pg.k = (pid[0] & kmask[0]) | (pid[1] & kmask[1]) | (pid[2] & kmask[2]) | (pid[3] & kmask[3]);
        pg.v = bt[min(tv * 4 + wu, last_page)];
    };
    // K: instruction i of wave w moves chunk 4 w + i of all 64 keys (four 256-byte runs, one per page);
    // V: wave w moves page w of the tile, whose [half][channel][8 keys] layout is the LDS layout (four 1 KiB runs)
    auto request_k = [&](int t, int mine) {
        const unsigned char* src = (const unsigned char*)kpool + ((int64_t)mine * hkv + g) * (int64_t)(D * PS * 2) + (wu * kPer) * 256 + kslot * 16;
        const unsigned dst = lds_address(k_lds) + (t % kKStages) * kTile + (wu * kPer) * 1024;
#pragma unroll
        for (int i = 0; i < kPer; ++i) load_to_lds(src + i * 256, dst + i * 1024);
    };
    auto request_v = [&](int stage, int pid) {
        const unsigned char* src = (const unsigned char*)vpool + ((int64_t)pid * hkv + g) * (int64_t)(D * PS * 2) + lane * 16;
        const unsigned dst = lds_address(v_lds) + stage * kTile + (wu * kPer) * 1024;
#pragma unroll
        for (int i = 0; i < kPer; ++i) load_to_lds(src + i * 1024, dst + i * 1024);
    };
    // slots of the session's last page that hold no token may contain anything (NaN included) and would poison
    // the value product even under a zero weight: once V(tv) has landed, zero them in LDS
    auto scrub_v = [&](int stage, int tv) {
        const int keep = it.ctx_all - (tv * BN + wu * PS);       // slots < keep of this wave's page hold tokens
        if (keep < PS) {                                         // uniform over the wave
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int half = i >> 1;                         // run i = 2 * half + (channels 64..127)
                u32x4* p = reinterpret_cast<u32x4*>(v_lds + stage * kTile + (wu * kPer + i) * 1024 + lane * 16);
                *p = tile32::keep_quads(*p, keep - half * 4, keep - 8 - half * 4);
            }
        }
    };

    const float sl2 = a.scale * kLog2e;
    float m = -INFINITY, lsum = 0.f;
    tile32::f32x16 o[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mb][i] = 0.f;
    const unsigned char* const k_lane = k_lds + n * 16 + hi * 1024;
    const unsigned char* const v_lane = v_lds + n * 16 + hi * 2048;

    // prologue: K(0) and K(1) requested and landed; the wait also tells the compiler that Q has arrived (it does
    // not see the direct loads and would otherwise wait for everything before each later use)
    Pages pg;
    pages_of(tb, tb, pg);
    request_k(0, pg.k);
    pages_of(tb + min(1, n_tiles - 1), tb, pg);
    request_k(1, pg.k);
    pages_of(tb + min(2, n_tiles - 1), tb, pg);                  // what iteration 0 requests: V(0) and K(2)
    AG_WAIT_VMCNT(0);
    __syncthreads();
    tile32::f32x16 sc[2];
    bf16x8 pa[4], pb[4];

    // Iteration t: S(t) from K(t); then P(t) side by side with O += V(t-1).P(t-1).  It starts by requesting V(t)
    // and K(t+2) and ends when V(t) and K(t+1) have landed.  Requests past the last tile repeat it into a buffer
    // nobody reads, so the loop has one shape; every wave runs all n_tiles + 1 iterations (the barriers are
    // workgroup-wide) and skips the pieces it does not need.
    auto iter = [&](int t, bf16x8 (&p_prev)[4], bf16x8 (&p_cur)[4]) {
        const int tv = min(t, n_tiles - 1);
        request_v(t & 1, pg.v);
        request_k(t + 2, pg.k);
        Pages nxt;
        pages_of(tb + min(t + 3, n_tiles - 1), tb + min(t + 1, n_tiles - 1), nxt);
        const bool do_sm = t < wave_tiles, do_pv = t >= 1 && t <= wave_tiles;
        const unsigned char* kb = k_lane + (t % kKStages) * kTile;
        const unsigned char* vb = v_lane + ((t + 1) & 1) * kTile;    // V(t-1)
        if (do_sm) {
            tile32::qk_tile(kb, qf, sc);
            if (t >= first_masked) {                 // the tile straddles this wave's diagonal
                const int kbase = (tb + t) * BN + hi * 4;
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kbase + b * 32 + (i >> 2) * 8 + (i & 3);
                        sc[b][i] = key <= qpos ? sc[b][i] : -INFINITY;
                    }
            }
        }
        tile32::softmax_and_value_product(do_sm, do_pv, vb, sc, sl2, m, lsum, p_prev, p_cur, o);
        AG_WAIT_VMCNT(kPer);
        scrub_v(t & 1, tb + tv);
        pg = nxt;
        __syncthreads();
    };
#pragma unroll 1
    for (int t = 0; t <= n_tiles; t += 2) {
        iter(t, pb, pa);
        if (t + 1 <= n_tiles) iter(t + 1, pa, pb);
    }
    AG_WAIT_VMCNT(0);                                // the last (redundant) tile requests still write to LDS

    // o[mb][q4 * 4 + e] is O^T[channel mb * 32 + q4 * 8 + hi * 4 + e][column n]; m is shared by the two lanes of a
    // column, l is the sum of both
    lsum += __shfl_xor(lsum, 32);
    if (on) {
        const int64_t slot = (((int64_t)a.cu_new[s] + t0 + token) * hq + (int64_t)g * G + col_head) * n_splits_max + it.split;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 x = {o[mb][q4 * 4], o[mb][q4 * 4 + 1], o[mb][q4 * 4 + 2], o[mb][q4 * 4 + 3]};
                *reinterpret_cast<f32x4*>(ws_o + slot * D + mb * 32 + q4 * 8 + hi * 4) = x;
            }
        if (hi == 0) { ws_ml[slot * 2] = m; ws_ml[slot * 2 + 1] = lsum; }
    }
}

// kSteps: the split size is 128 * kSteps keys.  R: column groups per wave.  kRows: the launch has rows items.
template <int kSteps, int R, bool kRows>
__global__ __launch_bounds__(256, R == 1 ? 4 : 2) void merged_split_kernel(AttnArgs a, float* __restrict__ ws_o,
                                                                           float* __restrict__ ws_ml,
                                                                           const int32_t* __restrict__ plan,
                                                                           int n_splits_max, int tq)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];     // kSmemBytes, or kRowsLds with rows items
    const int item = blockIdx.z;
    if (item >= plan[0]) return;
    const int32_t* e = plan + 4 + 4 * item;
    ItemCtx it;
    it.s = e[0]; it.t0 = e[1]; it.nt = e[2];
    const int kind = e[3];
    // Workgroups go to the XCDs round-robin in linear order (x fastest).  The split is blockIdx.x rotated by
    // head and session: short sessions only have the low split numbers, which would otherwise pile up on the
    // XCDs that draw them (see the decode step); rotating by the session, not the item, keeps the items of one
    // (session, KV head, split) on one XCD, whose L2 then serves what they fetch again.
    it.g = blockIdx.y;
    it.split = (int)((blockIdx.x + blockIdx.y + (unsigned)it.s) % gridDim.x);
    const int N = a.new_lens[it.s];
    it.P = a.prefix_lens ? a.prefix_lens[it.s] : 0;
    it.ctx_all = it.P + N;                           // slots below this hold tokens
    it.ctx = it.P + it.t0 + it.nt;                   // keys the item's last row may see
    it.part = part_tokens(it.ctx, 128 * kSteps);
    it.start = it.split * it.part;
    if (it.start >= it.ctx) return;                  // uniform over the workgroup
    if constexpr (kRows) {
        if (kind == kRowsItem) { rows_item<kSteps>(a, ws_o, ws_ml, n_splits_max, tq, it, smem); return; }
    }
    keys_item<kSteps, R>(a, ws_o, ws_ml, n_splits_max, tq, it, smem);
}

__global__ __launch_bounds__(128) void merged_merge_kernel(AttnArgs a, const float* __restrict__ ws_o,
                                                           const float* __restrict__ ws_ml,
                                                           const int32_t* __restrict__ row_ctx, int n_splits_max,
                                                           int split_tokens)
{
    const int64_t rh = blockIdx.x;                 // row * hq + head
    const int row = (int)(rh / a.hq);
    const int d = threadIdx.x;
    const int ctx = row_ctx[row];                  // as the split kernel cut the row's item
    const int part = part_tokens(ctx, split_tokens);
    const int n = (ctx + part - 1) / part;
    ((__bf16*)a.out)[rh * D + d] = (__bf16)merge_partials(ws_o, ws_ml, rh * n_splits_max, n, d);
}

inline int rows_per_group(int hq, int hkv) { return 16 / (hq / hkv); }

inline int choose_split(int64_t items, int hkv, int max_ctx, int largest)
{
    // As long as possible (every workgroup pays a fixed start-up) while the launch still has about eight
    // workgroups per CU, counting contexts at about 60 % of max_ctx: a queue that mixes a few long resume
    // prefixes with many shorter decode contexts is far below that estimate, and one round of long workgroups
    // balances badly.
    const int64_t want = 8 * 256;
    for (int split = largest; split > kMinSplit; split >>= 1) {
        const int64_t wgs = items * hkv * ((6 * (int64_t)max_ctx / 10 + split - 1) / split);
        if (wgs >= want) return split;
    }
    return kMinSplit;
}

struct Layout { size_t o_floats, ml_floats, plan_ints, row_ints; };
inline Layout layout(int total_rows, int hq, int max_ctx)
{
    const size_t nsm = (size_t)splits_for(max_ctx, kMinSplit);
    return {(size_t)total_rows * hq * nsm * D, (size_t)total_rows * hq * nsm * 2, 4 + 4 * (size_t)total_rows, (size_t)total_rows};
}

template <int kSteps, int R, bool kRows>
ag_status launch_one(dim3 grid, hipStream_t st, const AttnArgs& a, float* ws_o, float* ws_ml, const int32_t* plan, int nsm, int tq)
{
    constexpr int lds = kRows ? kRowsLds : kSmemBytes;
    if constexpr (kRows) {                  // more dynamic LDS than a kernel may use without being told so
        static std::atomic<bool> attr_set{false};
        if (!attr_set.load()) {
            ag_status e = hip_check(hipFuncSetAttribute((const void*)merged_split_kernel<kSteps, R, kRows>,
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, lds),
                                    "hipFuncSetAttribute(merged split)");
            if (e) return e;
            attr_set.store(true);
        }
    }
    hipLaunchKernelGGL((merged_split_kernel<kSteps, R, kRows>), grid, dim3(256), lds, st, a, ws_o, ws_ml, plan, nsm, tq);
    return AG_OK;
}

template <int R, bool kRows>
ag_status launch_split(int split, dim3 grid, hipStream_t st, const AttnArgs& a, float* ws_o, float* ws_ml,
                       const int32_t* plan, int nsm, int tq)
{
    switch (split) {
        case 2048:
            if constexpr (!kRows) return launch_one<16, R, false>(grid, st, a, ws_o, ws_ml, plan, nsm, tq);
            [[fallthrough]];     // not chosen for launches with rows items
        case 1024: return launch_one<8, R, kRows>(grid, st, a, ws_o, ws_ml, plan, nsm, tq);
        case 512:  return launch_one<4, R, kRows>(grid, st, a, ws_o, ws_ml, plan, nsm, tq);
        default:   return launch_one<2, R, kRows>(grid, st, a, ws_o, ws_ml, plan, nsm, tq);
    }
}

}  // namespace

size_t merged_workspace_bytes(int total_rows, int hq, int max_ctx)
{
    const Layout L = layout(total_rows, hq, max_ctx);
    return (L.o_floats + L.ml_floats + L.plan_ints + L.row_ints) * 4;
}

bool merged_mfma_supported(const AttnArgs& a)
{
    const int G = a.hq / a.c.hkv;
    return a.c.dtype == AG_BF16 && a.c.d == D && a.c.ps == PS && G <= 16 &&
           (((uintptr_t)a.q | (uintptr_t)a.c.k | (uintptr_t)a.c.v) % 16 == 0);
}

ag_status launch_merged_mfma(const AttnArgs& a, void* ws, hipStream_t st)
{
    if (a.total_rows <= 0) return AG_OK;
    const int tq = rows_per_group(a.hq, a.c.hkv);
    // A batch of decodes only (no session brings more rows than one group holds): one group per item, four
    // waves per SIMD.  Otherwise two groups per wave: keys items of up to 2 tq rows, and - once some session
    // may bring more than that - rows items of up to 8 tq rows.
    const int R = a.max_new > tq ? 2 : 1;
    const bool rows = a.max_new > R * tq;
    const int rk = R * tq, rw = rows ? 4 * R * tq : 0;
    // a session of N rows has at most N / (rows per full item) + 1 items, and every item has at least one row
    const int64_t items_max = std::min<int64_t>(a.total_rows, (int64_t)a.total_rows / (rw ? rw : rk) + a.batch);
    if (items_max > 65535 || a.c.hkv > 65535) { set_error("too many items (%lld) or KV heads for one launch grid", (long long)items_max); return AG_ERR_INVALID_ARG; }
    const int split = choose_split(items_max, a.c.hkv, a.max_ctx, rows ? 1024 : 2048);
    const int nsm = splits_for(a.max_ctx, split);
    const Layout L = layout(a.total_rows, a.hq, a.max_ctx);
    float* ws_o = (float*)ws;
    float* ws_ml = ws_o + L.o_floats;
    int32_t* plan = (int32_t*)(ws_ml + L.ml_floats);
    int32_t* row_ctx = plan + L.plan_ints;

    hipLaunchKernelGGL(merged_plan_kernel, dim3(1), dim3(256), 0, st, a.new_lens, a.prefix_lens, a.cu_new, a.batch,
                       a.total_rows, rk, rw, plan, row_ctx);
    ag_status e = hip_check(hipGetLastError(), "merged plan launch");
    if (e) return e;
    const dim3 grid(nsm, a.c.hkv, (unsigned)items_max);
    prof_before(st);
    if (R == 1) e = launch_split<1, false>(split, grid, st, a, ws_o, ws_ml, plan, nsm, tq);
    else if (!rows) e = launch_split<2, false>(split, grid, st, a, ws_o, ws_ml, plan, nsm, tq);
    else e = launch_split<2, true>(split, grid, st, a, ws_o, ws_ml, plan, nsm, tq);
    prof_after(st);
    if (e) return e;
    if ((e = hip_check(hipGetLastError(), "merged split launch"))) return e;
    hipLaunchKernelGGL(merged_merge_kernel, dim3((unsigned)((int64_t)a.total_rows * a.hq)), dim3(128), 0, st, a, ws_o, ws_ml,
                       row_ctx, nsm, split);
    return hip_check(hipGetLastError(), "merged merge launch");
}

}  // namespace ag
