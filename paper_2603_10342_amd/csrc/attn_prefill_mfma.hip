// Cold and resume prefill over a paged KV cache, bf16, head_dim 128, page 16
// (paper Sec. I and Sec. II-A: a cold prefill is full causal attention over
// the prompt; a resume prefill appends a chunk to a cached context, so row i
// of a session with P cached tokens sees keys 0 .. P + i.  Cold is P = 0.)
//
// A dense contraction, bound by the matrix cores: 4 * D flop per visible
// (query, key) pair and head.  One workgroup (4 waves) owns 128 consecutive
// query rows of one (session, query head); each wave owns 32 rows and keeps
// their Q in registers.  Keys and values are taken 64 at a time (4 pages) and
// staged through LDS:
//
//   S^T[key][query] = K[key][:] . Q[query][:]      2 x 8 MFMA 32x32x16
//   softmax weights per query column (running reference m, running sum l, exp2)
//   O^T[d][query]  += V^T[d][key] . P^T[key][query]  4 x 4 MFMA 32x32x16
//
// Computing the transposed score tile puts one query in one lane (plus its
// partner lane + 32), so the row max / sum need a single cross-lane step,
// and the 8 scores a lane holds for one k-step of the second product are
// already its B operand: P never leaves registers.  V pages are stored
// transposed with the slot order the score tile produces, so a value row
// copies straight into LDS.  LDS rows are padded so 16-byte operand reads
// are conflict free and every operand address is base + constant.
//
// The per-element softmax work on the vector ALUs is about as long as the
// matrix work (one exp per 512 flop), so the loop is software pipelined to
// run them side by side inside a wave.  Iteration t of a wave holds three
// independent pieces
//        S(t+1) = K(t+1).Q^T   (matrix)      P(t) = exp2(S(t) - m)   (vector)
//        O     += V(t-1).P(t-1) (matrix)
// in one basic block.  m is a reference, not the exact running maximum: O is
// rescaled only when a row's maximum has outgrown m by more than 2^8, which
// is decided before the block starts and takes a slower, ordered path, as do
// the tiles that straddle the diagonal (the only ones that need a mask).
// Tiles wholly above a wave's rows are skipped.
//
// Workgroups are numbered so that the XCD a workgroup lands on (id % 8) owns a
// contiguous range of KV heads, and inside it session-major, longest query
// tile first: the workgroups resident together read one session's K/V for one
// KV head, which then stays in that XCD's L2.
#include <atomic>

#include "ag_internal.h"

namespace ag {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int PS = 16;
constexpr int BM = 128;                 // query rows per workgroup
constexpr int BN = 64;                  // keys per tile
// LDS tiles with padded rows: a K row (one key, 256 B) is 272 B apart and a V^T row (one channel, 128 B) 144 B
// apart, so that the 16-byte operand reads of 16 neighbouring lanes fall in 16 different bank groups while
// every operand address is the lane's base plus a compile-time offset.
constexpr int kKRow = 272;
constexpr int kVRow = 144;
constexpr int kKTile = BN * kKRow;      // 17408
constexpr int kVTile = D * kVRow;       // 18432
constexpr int kLdsBytes = 2 * (kKTile + kVTile);   // two K tiles, then two V tiles: 71680
constexpr float kRescaleSlack = 8.0f;   // log2 units a row's maximum may grow before O is rescaled
constexpr float kLog2e = 1.4426950408889634f;

#ifndef AG_PREFILL_WAVES_PER_SIMD
#define AG_PREFILL_WAVES_PER_SIMD 2
#endif
#ifndef AG_PREFILL_AHEAD
#define AG_PREFILL_AHEAD 3
#endif

__device__ __forceinline__ u32x4 ld16g(const __bf16* p) { return *reinterpret_cast<const u32x4*>(p); }

// Elements 0..3 of u are slots j0 + {0..3}, elements 4..7 slots j0 + 8 + {0..3}: zero element e < 4 unless
// e < keep_lo and element 4 + e unless e < keep_hi.
__device__ __forceinline__ u32x4 keep_quads(u32x4 u, int keep_lo, int keep_hi)
{
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        u[w] &= ((2 * w < keep_lo) ? 0x0000FFFFu : 0u) | ((2 * w + 1 < keep_lo) ? 0xFFFF0000u : 0u);
        u[2 + w] &= ((2 * w < keep_hi) ? 0x0000FFFFu : 0u) | ((2 * w + 1 < keep_hi) ? 0xFFFF0000u : 0u);
    }
    return u;
}

// S^T tile (64 keys x 32 queries) = K tile . Q^T.  kb: this lane's base in a K tile (row n, half hi).
// Operand reads run kAhead matrix instructions ahead of their use; the two key blocks alternate so that
// neighbouring matrix instructions write different accumulators.
__device__ __forceinline__ void qk_tile(const unsigned char* kb, const bf16x8 (&qf)[8], f32x16 (&sc)[2])
{
    constexpr int kAhead = AG_PREFILL_AHEAD;
    bf16x8 opnd[kAhead + 1];
    auto operand = [&](int i) -> const unsigned char* { return kb + (i & 1) * 32 * kKRow + (i >> 1) * 32; };
#pragma unroll
    for (int i = 0; i < kAhead; ++i) opnd[i] = *reinterpret_cast<const bf16x8*>(operand(i));
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[b][i] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (i + kAhead < 16) opnd[(i + kAhead) % (kAhead + 1)] = *reinterpret_cast<const bf16x8*>(operand(i + kAhead));
        sc[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i % (kAhead + 1)], qf[i >> 1], sc[i & 1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// O^T (128 channels x 32 queries) += V^T tile . P^T.  vb: this lane's base in a V tile (row n, half hi).
__device__ __forceinline__ void pv_tile(const unsigned char* vb, const bf16x8 (&pb)[4], f32x16 (&o)[4])
{
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bf16x8 va = *reinterpret_cast<const bf16x8*>(vb + mb * 32 * kVRow + j * 32);
            o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[j], o[mb], 0, 0, 0);
        }
}

// Largest raw score among the 32 keys this lane holds for its query (its partner lane ^ 32 holds the other 32).
__device__ __forceinline__ float row_max(const f32x16 (&sc)[2])
{
    float mx = fmaxf(fmaxf(sc[0][0], sc[0][1]), sc[0][2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) mx = fmaxf(fmaxf(mx, sc[0][i]), sc[0][i + 1]);
    mx = fmaxf(fmaxf(mx, sc[0][15]), sc[1][0]);
#pragma unroll
    for (int i = 1; i < 15; i += 2) mx = fmaxf(fmaxf(mx, sc[1][i]), sc[1][i + 1]);
    mx = fmaxf(mx, sc[1][15]);
    return mx;
}

// P^T = exp2(S^T * sl2 - m) packed as the B operands of the four k-steps of the second product; adds to lsum.
__device__ __forceinline__ void exp_tile(const f32x16 (&sc)[2], float sl2, float m, float& lsum, bf16x8 (&pb)[4])
{
    float psum = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(sc[b][i], sl2, -m));
            psum += p;
            pb[b * 2 + (i >> 3)][i & 7] = (__bf16)p;
        }
    lsum += psum;
}

struct Stage {          // one thread's share of a K tile and a V tile on its way to LDS
    u32x4 k[4];
    u32x4 v[4];
};

__global__ __launch_bounds__(256, AG_PREFILL_WAVES_PER_SIMD) void prefill_mfma_kernel(AttnArgs a, int q_tiles,
                                                                                      int per_xcd, int64_t total_work)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // ---- which (session, head, query tile) ----
    const int xcd = blockIdx.x & 7, ord = blockIdx.x >> 3;
    const int64_t wk = (int64_t)xcd * per_xcd + ord;
    if (wk >= total_work) return;
    const int hkv = a.c.hkv, hq = a.hq, G = hq / hkv;
    // work order: KV head, then session, then query tile (longest first), then the G heads of the group
    const int per_sess = q_tiles * G;
    const int g = (int)(wk / ((int64_t)a.batch * per_sess));
    const int rem = (int)(wk % ((int64_t)a.batch * per_sess));
    const int s = rem / per_sess;
    const int qt = q_tiles - 1 - (rem % per_sess) / G;
    const int h = g * G + rem % G;

    const int N = a.new_lens[s];
    const int q0 = qt * BM;
    if (q0 >= N) return;
    const int P = a.prefix_lens ? a.prefix_lens[s] : 0;
    const int ctx = P + N;
    const int64_t t_base = (int64_t)a.cu_new[s] + q0;

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int n = lane & 31, hi = lane >> 5;
    const int rows_wg = min(BM, N - q0);            // valid query rows of this workgroup
    const int qrow0 = 32 * w;                       // first row of this wave inside the tile
    const int rows_w = max(0, min(32, rows_wg - qrow0));

    const int n_tiles = (P + q0 + rows_wg - 1) / BN + 1;                        // tiles the workgroup stages
    const int wave_tiles = rows_w > 0 ? (P + q0 + qrow0 + rows_w - 1) / BN + 1 : 0;   // tiles this wave uses
    const int first_masked = (P + q0 + qrow0 + 1) / BN;   // first tile holding a key this wave's row 0 may not see

    const __bf16* kpool = (const __bf16*)a.c.k;
    const __bf16* vpool = (const __bf16*)a.c.v;
    const int32_t* bt = a.bt + (int64_t)s * a.max_pages;
    const int last_page = (ctx - 1) >> 4;

    // ---- Q^T as B operand: column n = query row, k-step ks covers channels ks*16 + hi*8 .. +7 ----
    bf16x8 qf[8];
    {
        const int row = min(qrow0 + n, rows_wg - 1);
        const __bf16* qp = (const __bf16*)a.q + ((t_base + row) * hq + h) * D + hi * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    // ---- copy roles ----
    const int kslot = tid & 15, kc = tid >> 4;      // K: slot, chunk of 8 channels; pages 0..3 of the tile
    const int vd = tid & 127;                       // V: channel row, pages vpg0 and vpg0 + 2
    const int vpg0 = __builtin_amdgcn_readfirstlane(tid >> 7);   // uniform over a wave: keeps page ids scalar
    unsigned char* const k_lds = lds;                // K tile t lives at k_lds + (t & 1) * kKTile
    unsigned char* const v_lds = lds + 2 * kKTile;   // V tile t lives at v_lds + (t & 1) * kVTile

    // Physical pages of a tile, through scalar loads (the index is uniform).  They are fetched one iteration
    // before the tile's data is requested, so no data load ever waits for a block-table read.
    struct Pages { int k[4]; int v[2]; };
    auto pages_of = [&](int tk, int tv, Pages& pg) {
#pragma unroll
        for (int i = 0; i < 4; ++i) pg.k[i] = bt[min(tk * 4 + i, last_page)];
#pragma unroll
        for (int i = 0; i < 2; ++i) pg.v[i] = bt[min(tv * 4 + vpg0 + 2 * i, last_page)];
    };
    auto load_k = [&](const int (&pid)[4], Stage& st) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            st.k[i] = ld16g(kpool + ((int64_t)pid[i] * hkv + g) * (int64_t)(D * PS) + (kc * PS + kslot) * 8);
    };
    auto load_v = [&](int t, const int (&pid)[2], Stage& st) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = vpg0 + 2 * i;
            const __bf16* vp = vpool + (((int64_t)pid[i] * hkv + g) * D + vd) * PS;
            // a value-page row holds slots 0-3, 8-11 in its first 16 bytes and 4-7, 12-15 in the second
            u32x4 lo = ld16g(vp), hi8 = ld16g(vp + 8);
            const int keep = ctx - (t * BN + j * PS);           // slots < keep hold real tokens (uniform)
            if (keep < PS) {                                    // unwritten slots may hold anything
                lo = keep_quads(lo, keep, keep - 8);
                hi8 = keep_quads(hi8, keep - 4, keep - 12);
            }
            st.v[2 * i] = lo;
            st.v[2 * i + 1] = hi8;
        }
    };
    auto store_k = [&](int t, const Stage& st) {
        unsigned char* kb = k_lds + (t & 1) * kKTile;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(kb + (i * PS + kslot) * kKRow + kc * 16) = st.k[i];
    };
    auto store_v = [&](int t, const Stage& st) {
        unsigned char* vb = v_lds + (t & 1) * kVTile;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = vpg0 + 2 * i;
            *reinterpret_cast<u32x4*>(vb + vd * kVRow + (j * 2) * 16) = st.v[2 * i];
            *reinterpret_cast<u32x4*>(vb + vd * kVRow + (j * 2 + 1) * 16) = st.v[2 * i + 1];
        }
    };

    const float sl2 = a.scale * kLog2e;
    const int qpos = P + q0 + qrow0 + n;            // logical position of this lane's query
    float m = -INFINITY, lsum = 0.f;
    f32x16 o[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mb][i] = 0.f;

    const unsigned char* const k_lane = k_lds + n * kKRow + hi * 16;
    const unsigned char* const v_lane = v_lds + n * kVRow + hi * 16;

    // ---- prologue: K(0) into LDS ----
    Stage stg;
    Pages pg;
    pages_of(0, 0, pg);
    load_k(pg.k, stg);
    store_k(0, stg);
    pages_of(min(1, n_tiles - 1), 0, pg);            // what iteration 0 requests: K(1) and V(0)
    __syncthreads();
    f32x16 sc[2];
    bf16x8 pa[4], pb[4];

    // Iteration t of a wave: S(t) from K(t) (matrix); then P(t) = exp2(S(t) - m) (vector) side by side with
    // O += V(t-1).P(t-1) (matrix).  Global loads for K(t+1) and V(t) are issued at its start and land in LDS
    // at its end.  Every wave runs all n_tiles + 1 iterations (the barriers are workgroup-wide); the pieces a
    // wave does not need are skipped.
    auto iter = [&](int t, bf16x8 (&p_prev)[4], bf16x8 (&p_cur)[4]) {
        // Requests are unconditional (past the last tile they repeat it into a buffer nobody reads): the
        // loop body has one shape, so no wait is ever placed ahead of the compute on behalf of a skipped store.
        load_k(pg.k, stg);
        load_v(min(t, n_tiles - 1), pg.v, stg);
        pages_of(min(t + 2, n_tiles - 1), min(t + 1, n_tiles - 1), pg);   // for the next iteration's requests
        const bool do_sm = t < wave_tiles, do_pv = t >= 1 && t <= wave_tiles;
        const unsigned char* kb = k_lane + (t & 1) * kKTile;
        const unsigned char* vb = v_lane + ((t + 1) & 1) * kVTile;
        float mx = -INFINITY;
        if (do_sm) {
            qk_tile(kb, qf, sc);
            if (t >= first_masked) {                 // the tile straddles this wave's diagonal
                const int kbase = t * BN + hi * 4;
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kbase + b * 32 + (i >> 2) * 8 + (i & 3);
                        sc[b][i] = key <= qpos ? sc[b][i] : -INFINITY;
                    }
            }
            mx = row_max(sc) * sl2;                  // scale > 0: max and scaling commute
        }
        // m is shared by the two lanes of a query, but the test needs no exchange: if either lane's own
        // maximum outgrew m the whole wave takes the ordered path, which combines the two halves.
        const bool grow = __builtin_amdgcn_ballot_w64(mx > m + kRescaleSlack) != 0;   // uniform over the wave
        if (do_sm && do_pv && !grow) {
            // the common case: two independent pieces, interleaved by hand.  Step i issues the operand read
            // of matrix instruction i + kAhead, matrix instruction i, and the exp of scores 2i and 2i + 1;
            // the fences keep the compiler from regrouping them.  Neighbouring matrix instructions belong
            // to different accumulators.
            constexpr int kAhead = AG_PREFILL_AHEAD;
            bf16x8 opnd[kAhead + 1];
            auto operand = [&](int i) -> const unsigned char* {   // order (j, mb)
                return vb + (i & 3) * 32 * kVRow + (i >> 2) * 32;
            };
#pragma unroll
            for (int i = 0; i < kAhead; ++i) opnd[i] = *reinterpret_cast<const bf16x8*>(operand(i));
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (i + kAhead < 16) opnd[(i + kAhead) % (kAhead + 1)] = *reinterpret_cast<const bf16x8*>(operand(i + kAhead));
                o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i % (kAhead + 1)], p_prev[i >> 2], o[i & 3], 0, 0, 0);
                const int e = 2 * i;
                const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[e >> 4][e & 15], sl2, -m));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[e >> 4][(e & 15) + 1], sl2, -m));
                psum += p0 + p1;
                p_cur[e >> 3][e & 7] = (__bf16)p0;
                p_cur[e >> 3][(e & 7) + 1] = (__bf16)p1;
                __builtin_amdgcn_sched_barrier(0);
            }
            lsum += psum;
        } else {
            if (do_pv) pv_tile(vb, p_prev, o);
            if (do_sm) {
                if (grow) {
                    mx = fmaxf(mx, __shfl_xor(mx, 32));
                    const float m_new = fmaxf(m, mx);    // finite from tile 0 on: key 0 is visible to every row
                    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
                    lsum *= alpha;
#pragma unroll
                    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) o[mb][i] *= alpha;
                    m = m_new;
                }
                exp_tile(sc, sl2, m, lsum, p_cur);
            }
        }
        store_k(t + 1, stg);
        store_v(t, stg);
        __syncthreads();
    };

#pragma unroll 1
    for (int t = 0; t <= n_tiles; t += 2) {
        iter(t, pb, pa);
        if (t + 1 <= n_tiles) iter(t + 1, pa, pb);
    }

    // ---- normalise, transpose through LDS, store rows contiguously ----
    lsum += __shfl_xor(lsum, 32);
    const float inv = 1.0f / lsum;
    unsigned char* ob = lds + w * (32 * 256);       // this wave's [32 rows][128 ch] bf16, rows XOR-swizzled
    // (the barrier that closed the loop guarantees nobody still reads the K/V tiles)
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 x;
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = (__bf16)(o[mb][q4 * 4 + e] * inv);
            const int d = mb * 32 + q4 * 8 + hi * 4;            // 4 consecutive channels
            const int chunk = d >> 3;
            *reinterpret_cast<bf16x4*>(ob + n * 256 + ((chunk ^ (n & 15)) << 4) + (d & 7) * 2) = x;
        }
    __syncthreads();
    {
        const int c = lane & 15;
        __bf16* outp = (__bf16*)a.out;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int row = (lane >> 4) + 4 * k;
            if (row < rows_w) {
                const u32x4 x = *reinterpret_cast<const u32x4*>(ob + row * 256 + ((c ^ (row & 15)) << 4));
                *reinterpret_cast<u32x4*>(outp + ((t_base + qrow0 + row) * hq + h) * D + c * 8) = x;
            }
        }
    }
}

}  // namespace

bool prefill_mfma_supported(const AttnArgs& a)
{
    return a.c.dtype == AG_BF16 && a.c.d == D && a.c.ps == PS &&
           (((uintptr_t)a.q | (uintptr_t)a.out | (uintptr_t)a.c.k | (uintptr_t)a.c.v) % 16 == 0);
}

ag_status launch_prefill_mfma(const AttnArgs& a, hipStream_t st)
{
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load()) {
        ag_status e = hip_check(hipFuncSetAttribute((const void*)prefill_mfma_kernel,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes),
                                "hipFuncSetAttribute(prefill)");
        if (e) return e;
        attr_set.store(true);
    }
    const int q_tiles = (a.max_new + BM - 1) / BM;
    const int64_t total = (int64_t)a.batch * a.hq * q_tiles;
    const int64_t per_xcd = (total + 7) / 8;
    if (per_xcd * 8 > 0x7fffffff) { set_error("too many query tiles for one launch"); return AG_ERR_INVALID_ARG; }
    prof_before(st);
    hipLaunchKernelGGL(prefill_mfma_kernel, dim3((unsigned)(per_xcd * 8)), dim3(256), kLdsBytes, st, a, q_tiles,
                       (int)per_xcd, total);
    prof_after(st);
    return hip_check(hipGetLastError(), "prefill launch");
}

}  // namespace ag
