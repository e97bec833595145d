// One launch for the decode queue of the paper's scheduler: decodes and short resume prefills together
// (paper Sec. III-A: short resume prefills are merged with decodes to improve parallelism; Algorithm 1 admits
// a request to Q_D when it is a decode or no longer than B_prefill).  bf16, head_dim 128, page 16.
//
// A session brings N >= 0 new query rows at positions P .. P + N - 1 (a decode is N = 1) that attend causally
// to the session's keys: the semantics of the resume prefill.  The keys a session's rows may see are cut over
// workgroups, partial (m, l, O) per cut, merged in cut order, as in the decode step, because with few rows per
// session the launch is bound by reading K and V.  A session's rows are cut into items of two kinds:
//
//   keys item  one group of rows (a group is tq = 16 / G consecutive rows, G = query heads per KV head: its
//              tq x G (row, head) pairs fill the 16 columns of the matrix instruction that a decode leaves mostly
//              empty).  Work on it streams: the four waves of a workgroup split the keys, each K / V step
//              (32 keys) is loaded once into registers - the decode step's loop with a visibility limit per
//              column.  Bound by memory.
//   rows item  up to 8 groups of rows (32 rows at G = 4): four waves x 32 columns walk the same keys in the
//              prefill kernel's 64-key tiles, which the workgroup brings into LDS once (attn_tile32.h), so the
//              keys are fetched once per 8 groups.  Bound by the matrix cores.
//   A session has full rows items and a remainder that is a keys item if it fits one group, else one more rows
//   item; a decode, or any chunk of at most tq rows, is one keys item.
//
// The launch has exactly as many workgroups as the stream's CUs hold at once, and no planning launch: as in the
// decode step, the work of each kind is laid end to end - the keys items' (session, KV head) pairs in steps of 32
// keys, the rows items' (session, KV head, item) triples in tiles of 64 keys - and dealt in equal contiguous
// shares, W_T workgroups sharing the tiles and the other W_K the steps.  Every workgroup derives the totals, the
// two share sizes and its own starting point from the lengths on the device (a sum and a scan over the batch).
// W_T : W_K follows the cost of a tile against a step, so that both kinds end together; the tile workgroups come
// first in the grid, which spreads them over the CUs: a CU then holds matrix-bound and memory-bound work side by
// side for the whole launch.  A share is one segment (part of one pair or triple) or the end of one and the
// start of the next ones; each segment leaves a partial per (row, head), numbered by the workgroups the pair is
// cut over, and the first workgroup publishes what the merge kernel needs to count them.
#include <algorithm>
#include <atomic>

#include "attn_split_common.h"
#include "attn_tile32.h"
#include "lds_dma.h"

namespace ag {

namespace {

using namespace splitk;

constexpr int kMinSteps = kMinSplit / 32;       // a streaming share is at least this many steps (256 keys)
constexpr int kMinTiles = kMinSplit / 64;       // a tile share at least this many tiles (256 keys)
constexpr int kSmemBytes = 4 * 16 * D * 4 + 2 * 4 * 16 * 4;             // 33280: partials of four waves
constexpr int kRowsLds = (tile32::kKStages + 2) * tile32::kTile;        // 80 KiB: three K and two V tiles
// What the split of the workgroups between the two kinds of work rests on (measured with timestamps inside the
// kernel): a tile workgroup takes 2.1-2.2 us per 64-key tile; the streaming workgroups together move 369 steps of
// 32 keys per microsecond on the whole device (6.0 TB/s) however many they are, as long as they are enough to
// saturate the memory system; a single streaming workgroup cannot take a step in less than 0.57 us (what one CU
// can draw, for its two workgroups).
constexpr float kTileUs = 2.15f;
constexpr float kDeviceStepsPerUs = 369.0f;
constexpr float kStepUsAlone = 0.57f;

__device__ __forceinline__ int steps_of(int ctx) { return ctx > 0 ? (ctx + 31) >> 5 : 0; }
__device__ __forceinline__ int tiles_of(int ctx) { return ctx > 0 ? (ctx + 63) >> 6 : 0; }
// Segments a pair may be cut into: a pair has at most ceil(max_ctx / 32) steps (half as many tiles), and a share is
// at least kMinSteps steps (kMinTiles tiles).
inline int pieces_max(int max_ctx) { return (((max_ctx + 31) / 32) - 1) / kMinSteps + 2; }

// How a session's N rows are cut.  rk: rows of a full keys item; rw: rows of a full rows item, 0 if the launch
// has no rows items (then no session brings more than rk rows).
struct Cut {
    int n_rows_items;       // rows item j holds rows [j rw, min(N, (j + 1) rw))
    int k_t0, k_nt;         // rows of the keys item (none if k_nt = 0)
};
__device__ __forceinline__ Cut cut_of(int N, int rk, int rw)
{
    Cut c;
    if (rw == 0) { c.n_rows_items = 0; c.k_t0 = 0; c.k_nt = max(N, 0); return c; }
    const int full = N / rw, rem = N - full * rw;
    c.n_rows_items = full + (rem > rk ? 1 : 0);
    c.k_t0 = full * rw;
    c.k_nt = rem > rk ? 0 : rem;
    return c;
}
__device__ __forceinline__ int item_tiles(int N, int P, int rw, int j) { return tiles_of(P + min(N, (j + 1) * rw)); }
__device__ __forceinline__ int session_steps(const Cut& c, int P) { return c.k_nt > 0 ? steps_of(P + c.k_t0 + c.k_nt) : 0; }
__device__ __forceinline__ int session_tiles(const Cut& c, int N, int P, int rw)
{
    int t = 0;
    for (int j = 0; j < c.n_rows_items; ++j) t += item_tiles(N, P, rw, j);
    return t;
}

// What the merge kernel needs per query row: which kind of item holds it, the flat unit at which the item's
// pair starts for KV head 0, the distance to the next head's pair, and the pair's length.
struct RowInfo { int32_t kind, first, stride, n; };
enum { kKeysItem = 0, kRowsItem = 1 };

// What a segment needs to know about its item; uniform over the workgroup.
struct Seg {
    int s, g;               // session, KV head
    int t0, nt;             // the item's rows within the session's chunk
    int P, ctx_all, ctx;    // prefix, prefix + chunk (slots below hold tokens), keys the item's last row may see
    int u, k;               // the segment: units u .. u + k - 1 of the pair (steps of 32 keys, or tiles of 64)
    int piece;              // which of the pair's partials this segment leaves
};

// ---- a segment of a keys item: the decode step's loop with a visibility limit per column ----------------------
__device__ __forceinline__ void stream_segment(const AttnArgs& a, float* __restrict__ ws_o, float* __restrict__ ws_ml,
                                               int pmax, int tq, const Seg& sg, unsigned char* smem)
{
    float (*s_o)[16][D] = reinterpret_cast<float (*)[16][D]>(smem);                 // per wave, per column
    float (*s_m)[16] = reinterpret_cast<float (*)[16]>(smem + 4 * 16 * D * 4);
    float (*s_l)[16] = s_m + 4;

    const int s = sg.s, g = sg.g, t0 = sg.t0, nt = sg.nt, P = sg.P, ctx_all = sg.ctx_all, ctx = sg.ctx;
    const int hkv = a.c.hkv, hq = a.hq;
    const int G = hq / hkv;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, c = lane >> 4;
    // the four waves take contiguous quarters of the segment's steps
    const int per = (sg.k + 3) >> 2;
    const int my_u = sg.u + w * per;
    const int my_n = max(0, min(per, sg.k - w * per));

    const __bf16* kpool = (const __bf16*)a.c.k;
    const __bf16* vpool = (const __bf16*)a.c.v;

    // column r = (row r / G of the item, head r % G of the KV head's group); columns without a row carry a zero
    // query and the visibility of the item's last row
    const int col_row = r / G, col_head = r - col_row * G;
    const bool on = col_row < tq && col_row < nt;
    const int pos = P + t0 + (on ? col_row : nt - 1);
    bf16x8 qf[4];
    {
        const int64_t q_row = (int64_t)a.cu_new[s] + t0 + (on ? col_row : 0);
        const __bf16* qrow = (const __bf16*)a.q + (q_row * hq + (int64_t)g * G + col_head) * D + c * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 x = ld16(qrow + kk * 32);
            if (!on) x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qf[kk] = x;
        }
    }

    const int last_lp = ((ctx + PS - 1) >> 4) - 1;
    const float sl2 = a.scale * kLog2e;
    float m = -INFINITY, lsum = 0.0f;
    f32x4 o[8];
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // operand addressing as in the decode step: score row r is slot (r & 7) of page (r >> 3) of the step, the
    // second score product takes slots 8..15; lane group c owns the 8 keys of value chunk (c & 1) of page (c >> 1)
    const int k_pg = r >> 3;
    const int k_off = (c * PS + (r & 7)) * 8;
    const int v_pg = c >> 1;
    const int v_off = ((c & 1) * D + r) * 8;

    // the wave's steps in runs of 32 (64 pages: one physical page id per lane)
#pragma unroll 1
    for (int run = 0; run < my_n; run += 32) {
        const int my_pid = a.bt[(int64_t)s * a.max_pages + min(2 * (my_u + run) + lane, last_lp)];
        const int n_here = min(32, my_n - run);
#pragma unroll 1
        for (int st = 0; st < n_here; ++st) {
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
                __builtin_amdgcn_sched_barrier(0);       // all 16 loads in flight before anything waits
            }
            const int tok0 = (my_u + run + st) * 32;
            const int tokb = tok0 + (c >> 1) * PS + (c & 1) * 4;
            f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k1[kk], qf[kk], s1, 0, 0, 0);
                s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k2[kk], qf[kk], s2, 0, 0, 0);
            }
            // s1[i]: key tokb + i, s2[i]: key tokb + 8 + i, of column r
            const int keep = pos + 1 - tokb;         // key tokb + i is visible to this column iff i < keep
            float xs[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xs[i] = (i < keep) ? s1[i] * sl2 : -INFINITY;
                xs[4 + i] = (8 + i < keep) ? s2[i] * sl2 : -INFINITY;
            }
            float mx = fmaxf(fmaxf(fmaxf(xs[0], xs[1]), fmaxf(xs[2], xs[3])), fmaxf(fmaxf(xs[4], xs[5]), fmaxf(xs[6], xs[7])));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m, mx);
            // a column may see none of this wave's keys so far (its row lies before them): keep the exponents finite
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m - m_ref);
            float psum = 0.f;
            bf16x8 pb;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float p = __builtin_amdgcn_exp2f(xs[e] - m_ref);
                psum += p;
                pb[e] = (__bf16)p;
            }
            lsum = lsum * alpha + psum;
            m = m_new;
            if (tok0 + 32 > ctx_all) {               // slots past the session's last token may hold anything, NaN included
                const int keep_v = ctx_all - tokb;
#pragma unroll
                for (int mb = 0; mb < 8; ++mb) x.v[mb] = keep_quads(x.v[mb], keep_v, keep_v - 8);
            }
#pragma unroll
            for (int mb = 0; mb < 8; ++mb) {
                o[mb] *= alpha;
                o[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.v[mb], pb, o[mb], 0, 0, 0);
            }
        }
    }

    // the four waves' partials through LDS; o[mb][i] is O^T[d = mb*16 + c*4 + i][column r]
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) *reinterpret_cast<f32x4*>(&s_o[w][r][mb * 16 + c * 4]) = o[mb];
    if (c == 0) { s_m[w][r] = m; s_l[w][r] = lsum; }
    __syncthreads();
    if (sg.piece < pmax) {
        const int n_cols = min(tq, nt) * G;
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
            const int64_t slot = (((int64_t)a.cu_new[s] + t0 + crow) * hq + (int64_t)g * G + chead) * pmax + sg.piece;
            ws_o[slot * D + d] = acc;
            if (d == 0) { ws_ml[slot * 2] = ms; ws_ml[slot * 2 + 1] = lt; }
        }
    }
    __syncthreads();                                         // the next segment writes the same LDS
}

// ---- a segment of a rows item: four waves x 32 columns over the same keys, in the prefill kernel's tiles --------
// Wave w holds column groups 2w and 2w + 1 of the item (group j = tokens j * tq .. + tq - 1, column r of a group =
// token r / G, head r % G): 32 columns, the B operand of the 32x32x16 products.  The segment's keys are walked in
// tiles of 64 (four pages) that the workgroup brings into LDS by direct global-to-LDS loads - three K stages,
// two V stages, tile layouts and software pipeline as in the prefill kernel (attn_tile32.h) - and every wave
// writes the partial (m, l, O) of its columns for the segment straight to the workspace.
__device__ __forceinline__ void tile_segment(const AttnArgs& a, float* __restrict__ ws_o, float* __restrict__ ws_ml,
                                             int pmax, int tq, const Seg& it, unsigned char* lds)
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

    // key tiles of the segment: tiles tb .. tb + n_tiles - 1 of the keys the item's last row may see
    const int tb = it.u, n_tiles = it.k;                          // >= 1

    // this lane's column; columns without a row carry the item's last row (their results are not stored)
    const int r = n & 15;
    const int col_row = r / G, col_head = r - col_row * G;
    const int token = (2 * w + (n >> 4)) * tq + col_row;
    const bool on = col_row < tq && token < nt;
    const int row = on ? token : nt - 1;
    const int qpos = P + t0 + row;                               // logical position of this lane's query
    const int w_first = 2 * w * tq;                              // the wave's first token
    const int w_last = min(nt, w_first + 2 * tq) - 1;            // ... and last
    // tiles of the segment this wave uses (none if it has no rows, or if the segment lies above all of them), and the
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
    if (on && it.piece < pmax) {
        const int64_t slot = (((int64_t)a.cu_new[s] + t0 + token) * hq + (int64_t)g * G + col_head) * pmax + it.piece;
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

// kRows: the launch has rows items.
// hdr[0], hdr[1]: the share sizes (steps per streaming workgroup, tiles per tile workgroup), for the merge kernel.
template <bool kRows>
__global__ __launch_bounds__(256, 2) void merged_split_kernel(AttnArgs a, int32_t* __restrict__ hdr,
                                                                           RowInfo* __restrict__ row_info,
                                                                           float* __restrict__ ws_o,
                                                                           float* __restrict__ ws_ml, int pmax,
                                                                           int tq, int rk, int rw, float steps_per_us)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];     // kSmemBytes, or kRowsLds with rows items
    // The plan's few words of LDS lie in the same buffer as the segments' data (two workgroups of 80 KiB fill a
    // CU's LDS exactly); a barrier separates the plan's last read from the first segment.
    int (*s_red)[4] = reinterpret_cast<int (*)[4]>(smem);                     // [2][4]
    int* s_start = reinterpret_cast<int*>(smem) + 8;    // session holding the workgroup's first unit, units before it, N, P

    const int B = a.batch, hkv = a.c.hkv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int W = gridDim.x;
    auto lengths = [&](int s, int& N, int& P) {
        N = s < B ? a.new_lens[s] : 0;
        P = (s < B && a.prefix_lens) ? a.prefix_lens[s] : 0;
    };

    // ---- the plan: totals of both kinds, the split of the workgroups, the two share sizes, where this
    // workgroup's share starts.  One pass over the lengths when the batch fits it (the scan's totals are the
    // totals); a larger batch is summed first. ----
    int tot_k = 0, tot_t = 0;
    if (B > 256) {
        int lk = 0, lt = 0;
        for (int s = tid; s < B; s += 256) {
            int N, P;
            lengths(s, N, P);
            const Cut c = cut_of(N, rk, rw);
            lk += session_steps(c, P);
            if (kRows) lt += session_tiles(c, N, P, rw);
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { lk += __shfl_xor(lk, d); lt += __shfl_xor(lt, d); }
        if (lane == 0) { s_red[0][w] = lk; s_red[1][w] = lt; }
        __syncthreads();
        tot_k = s_red[0][0] + s_red[0][1] + s_red[0][2] + s_red[0][3];
        tot_t = s_red[1][0] + s_red[1][1] + s_red[1][2] + s_red[1][3];
        __syncthreads();
    }
    const bool first_wg = blockIdx.x == 0;
    int F_K = 0, F_T = 0, W_T = 0, q_K = kMinSteps, q_T = kMinTiles, me = 0, f0 = 0, f1 = 0;
    bool tiles = false, active = false;
    if (tid == 0) s_start[0] = B;           // (no session: nothing runs; cannot happen while the lengths stand still)
    {
        int carry_k = 0, carry_t = 0;       // units of the sessions before this pass of 256
        for (int s0 = 0; s0 < B; s0 += 256) {
            const int s = s0 + tid;
            int N, P;
            lengths(s, N, P);
            const Cut c = cut_of(N, rk, rw);
            const int nk = session_steps(c, P), nt = kRows ? session_tiles(c, N, P, rw) : 0;
            int ik = nk, it = nt;           // inclusive scans over the wave
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int tk = __shfl_up(ik, d), tt = __shfl_up(it, d);
                if (lane >= d) { ik += tk; it += tt; }
            }
            if (lane == 63) { s_red[0][w] = ik; s_red[1][w] = it; }
            __syncthreads();
            int off_k = 0, off_t = 0;
            for (int ww = 0; ww < w; ++ww) { off_k += s_red[0][ww]; off_t += s_red[1][ww]; }
            const int pass_k = s_red[0][0] + s_red[0][1] + s_red[0][2] + s_red[0][3];
            const int pass_t = s_red[1][0] + s_red[1][1] + s_red[1][2] + s_red[1][3];
            if (s0 == 0) {                  // every value here is uniform over the workgroup
                if (B <= 256) { tot_k = pass_k; tot_t = pass_t; }
                F_K = hkv * tot_k;
                F_T = kRows ? hkv * tot_t : 0;
                if (F_K + F_T == 0) return;
                // W_T so that both kinds end together.  While the streaming workgroups left over still saturate
                // the memory system, the steps take F_K / steps_per_us whatever their number, and the tiles get
                // the workgroups that finish them in that time; otherwise every workgroup is busy for the whole
                // launch, and the workgroups are divided as the slot-times of the two kinds.
                if (F_T > 0) {
                    if (F_K == 0) {
                        W_T = W;
                    } else {
                        const float tile_us = kTileUs * (float)F_T;
                        float wt = tile_us * steps_per_us / (float)F_K;
                        if ((float)W - wt < steps_per_us * kStepUsAlone) wt = (float)W * tile_us / (tile_us + kStepUsAlone * (float)F_K);
                        W_T = max(1, min(W - 1, (int)(wt + 0.5f)));
                    }
                }
                const int W_K = W - W_T;
                if (F_K > 0) q_K = max(kMinSteps, (F_K + W_K - 1) / W_K);
                if (F_T > 0) q_T = max(kMinTiles, (F_T + W_T - 1) / W_T);
                if (first_wg && tid == 0) { hdr[0] = q_K; hdr[1] = q_T; }
                // this workgroup's share: the tile workgroups come first in the grid
                tiles = (int)blockIdx.x < W_T;
                me = tiles ? blockIdx.x : blockIdx.x - W_T;       // number among the workgroups of its kind
                const int q = tiles ? q_T : q_K, F = tiles ? F_T : F_K;
                f0 = me * q;
                f1 = min(f0 + q, F);
                active = f0 < F;
                if (!active && !first_wg) return;
            }
            const int excl_k = carry_k + off_k + ik - nk, excl_t = carry_t + off_t + it - nt;
            const int mine = tiles ? nt : nk, excl = tiles ? excl_t : excl_k;
            if (active && mine > 0 && hkv * excl <= f0 && f0 < hkv * (excl + mine)) {
                s_start[0] = s; s_start[1] = excl; s_start[2] = N; s_start[3] = P;
            }
            if (first_wg && s < B) {        // the first workgroup also publishes the rows' plan for the merge kernel
                const int row0 = a.cu_new[s];
                int acc = 0;                // tiles of the session's earlier rows items
                for (int j = 0; j < c.n_rows_items; ++j) {
                    const int tj = item_tiles(N, P, rw, j);
                    for (int x = j * rw; x < min(N, (j + 1) * rw); ++x)
                        if (row0 + x < a.total_rows) row_info[row0 + x] = RowInfo{kRowsItem, hkv * excl_t + acc, nt, tj};
                    acc += tj;
                }
                for (int x = c.k_t0; x < c.k_t0 + c.k_nt; ++x)
                    if (row0 + x < a.total_rows) row_info[row0 + x] = RowInfo{kKeysItem, hkv * excl_k, nk, nk};
            }
            __syncthreads();
            carry_k += pass_k;
            carry_t += pass_t;
            if (!first_wg && hkv * (tiles ? carry_t : carry_k) > f0) break;       // found (uniform)
        }
    }
    if (!active) return;
    int s = s_start[0];
    int base = hkv * s_start[1];            // flat unit at which session s starts
    int N = s_start[2], P = s_start[3];
    Cut c = cut_of(N, rk, rw);
    __syncthreads();                        // the segments reuse the plan's LDS

    if (!tiles) {
        // ---- streaming share: segments of (session, KV head) pairs, n steps each ----
        int n = session_steps(c, P);
        int g = (f0 - base) / n;
        int u = (f0 - base) - g * n;
        for (int f = f0; f < f1 && s < B;) {                 // one segment per pass; every value here is uniform
            const int k = min(n - u, f1 - f);
            if (k <= 0) break;                               // (only if the lengths changed under the kernel: never spin)
            Seg sg;
            sg.s = s; sg.g = g; sg.t0 = c.k_t0; sg.nt = c.k_nt; sg.P = P; sg.ctx_all = P + N; sg.ctx = P + c.k_t0 + c.k_nt;
            sg.u = u; sg.k = k;
            sg.piece = me - (base + g * n) / q_K;            // the pair's partials are numbered from its first workgroup
            stream_segment(a, ws_o, ws_ml, pmax, tq, sg, smem);
            f += k;
            u += k;
            if (u == n) {                                    // on to the next pair
                u = 0;
                if (++g == hkv) {
                    g = 0;
                    base += hkv * n;
                    do {
                        ++s;
                        lengths(s, N, P);
                        c = cut_of(N, rk, rw);
                        n = session_steps(c, P);
                    } while (s < B && n == 0);
                }
            }
        }
    } else if constexpr (kRows) {
        // ---- tile share: segments of (session, KV head, rows item) triples; a session has n tiles per KV head ----
        int n = session_tiles(c, N, P, rw);
        int g = (f0 - base) / n;
        int u = (f0 - base) - g * n;        // first tile inside (s, g): find the item it falls in
        int j = 0, before = 0;              // ... and the tiles of the items before it
        for (;;) {
            const int tj = item_tiles(N, P, rw, j);
            if (u < tj || j + 1 >= c.n_rows_items) break;
            u -= tj; before += tj; ++j;
        }
        for (int f = f0; f < f1 && s < B;) {
            const int tj = item_tiles(N, P, rw, j);
            const int k = min(tj - u, f1 - f);
            if (k <= 0) break;
            Seg sg;
            sg.s = s; sg.g = g; sg.t0 = j * rw; sg.nt = min(rw, N - j * rw); sg.P = P; sg.ctx_all = P + N;
            sg.ctx = P + sg.t0 + sg.nt;
            sg.u = u; sg.k = k;
            sg.piece = me - (base + g * n + before) / q_T;
            tile_segment(a, ws_o, ws_ml, pmax, tq, sg, smem);
            f += k;
            u += k;
            if (u == tj) {                                   // on to the next item, head, session
                u = 0;
                before += tj;
                if (++j == c.n_rows_items) {
                    j = 0;
                    before = 0;
                    if (++g == hkv) {
                        g = 0;
                        base += hkv * n;
                        do {
                            ++s;
                            lengths(s, N, P);
                            c = cut_of(N, rk, rw);
                            n = session_tiles(c, N, P, rw);
                        } while (s < B && n == 0);
                    }
                }
            }
        }
    }
}

// Two (row, head) pairs per workgroup: the pair's partials are those of the workgroups its units were dealt to.
__global__ __launch_bounds__(256) void merged_merge_kernel(AttnArgs a, const int32_t* __restrict__ hdr,
                                                           const RowInfo* __restrict__ row_info,
                                                           const float* __restrict__ ws_o,
                                                           const float* __restrict__ ws_ml, int pmax)
{
    const int64_t rh = (int64_t)blockIdx.x * 2 + (threadIdx.x >> 7);        // row * hq + head
    if (rh >= (int64_t)a.total_rows * a.hq) return;
    const int row = (int)(rh / a.hq), head = (int)(rh - (int64_t)row * a.hq);
    const int d = threadIdx.x & 127;
    const RowInfo ri = row_info[row];
    const int q = max(1, hdr[ri.kind == kRowsItem ? 1 : 0]);
    const int first = ri.first + (head / (a.hq / a.c.hkv)) * ri.stride;
    const int pieces = min(pmax, (first + ri.n - 1) / q - first / q + 1);
    ((__bf16*)a.out)[rh * D + d] = (__bf16)merge_partials(ws_o, ws_ml, rh * pmax, pieces, d);
}

inline int rows_per_group(int hq, int hkv) { return 16 / (hq / hkv); }

struct Layout { size_t o_floats, ml_floats, hdr_ints, row_ints; };
inline Layout layout(int total_rows, int hq, int max_ctx)
{
    const size_t pm = (size_t)pieces_max(max_ctx);
    return {(size_t)total_rows * hq * pm * D, ((size_t)total_rows * hq * pm * 2 + 3) & ~(size_t)3, 4, 4 * (size_t)total_rows};
}

template <bool kRows>
ag_status launch_split(int n_wgs, hipStream_t st, const AttnArgs& a, int32_t* hdr, RowInfo* row_info, float* ws_o,
                       float* ws_ml, int pmax, int tq, int rk, int rw, float steps_per_us)
{
    constexpr int lds = kRows ? kRowsLds : kSmemBytes;
    if constexpr (kRows) {                  // more dynamic LDS than a kernel may use without being told so
        static std::atomic<bool> attr_set{false};
        if (!attr_set.load()) {
            ag_status e = hip_check(hipFuncSetAttribute((const void*)merged_split_kernel<kRows>,
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, lds),
                                    "hipFuncSetAttribute(merged split)");
            if (e) return e;
            attr_set.store(true);
        }
    }
    hipLaunchKernelGGL((merged_split_kernel<kRows>), dim3((unsigned)n_wgs), dim3(256), lds, st, a, hdr, row_info, ws_o,
                       ws_ml, pmax, tq, rk, rw, steps_per_us);
    return AG_OK;
}

}  // namespace

size_t merged_workspace_bytes(int total_rows, int hq, int max_ctx)
{
    const Layout L = layout(total_rows, hq, max_ctx);
    return (L.o_floats + L.ml_floats + L.hdr_ints + L.row_ints) * 4;
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
    // Keys items hold one group of rows (tq: a decode, or a chunk that fits the 16 columns with its heads); once
    // some session may bring more, there are rows items of up to 8 groups.  (Keys items of two groups - the
    // streaming loop with twice the arithmetic per step for every item, decodes included - measured 146 against
    // 127 us on a queue of 64 decodes and 8 chunks of 8 rows.)
    const bool rows = a.max_new > tq;
    const int rk = tq, rw = rows ? 8 * tq : 0;
    const Layout L = layout(a.total_rows, a.hq, a.max_ctx);
    const int pmax = pieces_max(a.max_ctx);
    float* ws_o = (float*)ws;
    float* ws_ml = ws_o + L.o_floats;
    int32_t* hdr = (int32_t*)(ws_ml + L.ml_floats);
    RowInfo* row_info = (RowInfo*)(hdr + L.hdr_ints);
    // As many workgroups as the stream's CUs hold at once (paper Sec. III-C: the decode queue runs on a partition).
    // The steps the stream's CUs can move per microsecond: the device's rate, or what its CUs can draw if that
    // is less (two workgroups per CU at 0.57 us a step each).
    const int cus = stream_cus(st);
    const int n_wgs = 2 * cus;      // equal shares: as few workgroups as fill every CU evenly, as in the decode step
    const float steps_per_us = std::min(kDeviceStepsPerUs * (float)device_cus() / 256.0f, 2.0f * (float)cus / kStepUsAlone);

    prof_before(st);
    ag_status e;
    if (!rows) e = launch_split<false>(n_wgs, st, a, hdr, row_info, ws_o, ws_ml, pmax, tq, rk, rw, steps_per_us);
    else e = launch_split<true>(n_wgs, st, a, hdr, row_info, ws_o, ws_ml, pmax, tq, rk, rw, steps_per_us);
    prof_after(st);
    if (e) return e;
    if ((e = hip_check(hipGetLastError(), "merged split launch"))) return e;
    const int64_t pairs = (int64_t)a.total_rows * a.hq;
    hipLaunchKernelGGL(merged_merge_kernel, dim3((unsigned)((pairs + 1) / 2)), dim3(256), 0, st, a, hdr, row_info, ws_o, ws_ml, pmax);
    return hip_check(hipGetLastError(), "merged merge launch");
}

}  // namespace ag
