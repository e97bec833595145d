// Cold and resume prefill over a paged KV cache, bf16, head_dim 128, page 16
// (paper Sec. I and Sec. II-A: a cold prefill is full causal attention over
// the prompt; a resume prefill appends a chunk to a cached context, so row i
// of a session with P cached tokens sees keys 0 .. P + i.  Cold is P = 0.)
//
// A dense contraction, bound by the matrix cores: 4 * D flop per visible
// (query, key) pair and head.  One workgroup (4 waves) owns 128 consecutive
// query rows of one (session, query head); each wave owns 32 rows and keeps
// their Q in registers.  Keys and values are taken 64 at a time (4 pages),
// staged through LDS (double buffered, one barrier per tile):
//
//   S^T[key][query] = K[key][:] . Q[query][:]      2 x 8 MFMA 32x32x16
//   streaming softmax per query column (running max / sum, exp2)
//   O^T[d][query]  += V^T[d][key] . P^T[key][query]  4 x 4 MFMA 32x32x16
//
// Computing the transposed score tile puts one query in one lane (plus its
// partner lane + 32), so the row max / sum need a single cross-lane step,
// and the 8 scores a lane holds for one k-step of the second product are
// already the B operand: P never leaves registers.  V pages are stored
// transposed ([d][slot]); the copy into LDS orders the keys of each 16-byte
// chunk to match that operand.  Both LDS tiles are XOR-swizzled by row so
// the 16-byte operand reads are conflict free.
//
// Tiles wholly above a wave's rows are skipped; only tiles that straddle the
// diagonal are masked.  Workgroups are numbered so that the XCD a workgroup
// lands on (id % 8) owns a contiguous range of KV heads, keeping a session's
// K/V for that head in one L2, and within it the longest query tiles go first.
#include <atomic>

#include "ag_internal.h"

namespace ag {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

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
constexpr int kStage = kKTile + kVTile; // 35840
constexpr int kLdsBytes = 2 * kStage;   // 71680: two workgroups per CU fit in 160 KiB
constexpr float kRescaleSlack = 8.0f;   // log2 units a row's maximum may grow before O is rescaled
constexpr float kLog2e = 1.4426950408889634f;

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

struct Stage {          // one thread's share of a K tile and a V tile on its way to LDS
    u32x4 k[4];
    u32x4 v[4];
};

__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(AttnArgs a, int q_tiles, int per_xcd, int64_t total_work)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // ---- which (session, head, query tile) ----
    const int xcd = blockIdx.x & 7, ord = blockIdx.x >> 3;
    const int64_t wk = (int64_t)xcd * per_xcd + ord;
    if (wk >= total_work) return;
    const int hkv = a.c.hkv, hq = a.hq, G = hq / hkv;
    // work order: KV head, then session, then query tile (longest first), then the G heads of the group, so
    // that the workgroups resident on one XCD at a time read the same session's K/V for one KV head: it stays in L2
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

    const int n_tiles = (P + q0 + rows_wg - 1) / BN + 1;
    const int wave_tiles = rows_w > 0 ? (P + q0 + qrow0 + rows_w - 1) / BN + 1 : 0;
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
    const int vd = tid & 127, vpg0 = tid >> 7;      // V: channel row, pages vpg0 and vpg0 + 2

    auto load_tile = [&](int t, Stage& st) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t page = bt[min(t * 4 + i, last_page)];
            st.k[i] = ld16g(kpool + (page * hkv + g) * (int64_t)(D * PS) + (kc * PS + kslot) * 8);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = vpg0 + 2 * i;
            const int64_t page = bt[min(t * 4 + j, last_page)];
            const __bf16* vp = vpool + ((page * hkv + g) * D + vd) * PS;
            // a value-page row holds slots 0-3, 8-11 in its first 16 bytes and 4-7, 12-15 in the second
            u32x4 lo = ld16g(vp), hi8 = ld16g(vp + 8);
            const int keep = ctx - (t * BN + j * PS);           // slots < keep hold real tokens
            if (keep < PS) {                                    // unwritten slots may hold anything
                lo = keep_quads(lo, keep, keep - 8);
                hi8 = keep_quads(hi8, keep - 4, keep - 12);
            }
            st.v[2 * i] = lo;
            st.v[2 * i + 1] = hi8;
        }
    };
    auto store_tile = [&](int buf, const Stage& st) {
        unsigned char* kb = lds + buf * kStage;
        unsigned char* vb = kb + kKTile;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(kb + (i * PS + kslot) * kKRow + kc * 16) = st.k[i];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = vpg0 + 2 * i;
            *reinterpret_cast<u32x4*>(vb + vd * kVRow + (j * 2) * 16) = st.v[2 * i];
            *reinterpret_cast<u32x4*>(vb + vd * kVRow + (j * 2 + 1) * 16) = st.v[2 * i + 1];
        }
    };

    const float sl2 = a.scale * kLog2e;
    float m = -INFINITY, lsum = 0.f;
    f32x16 o[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mb][i] = 0.f;

    Stage stg;
    load_tile(0, stg);
    store_tile(0, stg);
    __syncthreads();

    const int qpos = P + q0 + qrow0 + n;            // logical position of this lane's query

#pragma unroll 1
    for (int t = 0; t < n_tiles; ++t) {
        const bool more = t + 1 < n_tiles;
        if (more) load_tile(t + 1, stg);

        if (t < wave_tiles) {
            const unsigned char* kb = lds + (t & 1) * kStage + n * kKRow + hi * 16;
            const unsigned char* vb = lds + (t & 1) * kStage + kKTile + n * kVRow + hi * 16;
            f32x16 sc[2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
#pragma unroll
                for (int i = 0; i < 16; ++i) sc[b][i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 ka = *reinterpret_cast<const bf16x8*>(kb + b * 32 * kKRow + ks * 32);
                    sc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[ks], sc[b], 0, 0, 0);
                }
            }
            // sc[b][i] is key t*64 + b*32 + (i/4)*8 + hi*4 + i%4 against query n (raw dot products)
            if (t >= first_masked) {
                const int kbase = t * BN + hi * 4;
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kbase + b * 32 + (i >> 2) * 8 + (i & 3);
                        sc[b][i] = key <= qpos ? sc[b][i] : -INFINITY;
                    }
            }
            float mx = fmaxf(fmaxf(sc[0][0], sc[0][1]), sc[0][2]);
#pragma unroll
            for (int i = 3; i < 15; i += 2) mx = fmaxf(fmaxf(mx, sc[0][i]), sc[0][i + 1]);
            mx = fmaxf(fmaxf(mx, sc[0][15]), sc[1][0]);
#pragma unroll
            for (int i = 1; i < 15; i += 2) mx = fmaxf(fmaxf(mx, sc[1][i]), sc[1][i + 1]);
            mx = fmaxf(mx, sc[1][15]);
            mx = fmaxf(mx, __shfl_xor(mx, 32)) * sl2;       // scale > 0: max and scaling commute
            // The reference m only has to stay within a few powers of two of the row maximum (any shift
            // cancels in O / l), so O is rescaled only when some row's maximum outgrew m by more than the
            // slack; until then weights may reach 2^slack, harmless in fp32 and bf16.
            if (__builtin_amdgcn_ballot_w64(mx > m + kRescaleSlack) != 0) {       // uniform over the wave
                const float m_new = fmaxf(m, mx);           // finite from tile 0 on: key 0 is visible to every row
                const float alpha = __builtin_amdgcn_exp2f(m - m_new);
                lsum *= alpha;
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[mb][i] *= alpha;
                m = m_new;
            }
            float psum = 0.f;
            bf16x8 pb[4];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sc[b][i], sl2, -m));
                    psum += p;
                    pb[b * 2 + (i >> 3)][i & 7] = (__bf16)p;
                }
            lsum += psum;
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bf16x8 va = *reinterpret_cast<const bf16x8*>(vb + mb * 32 * kVRow + j * 32);
                    o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[j], o[mb], 0, 0, 0);
                }
            }
        }

        if (more) store_tile((t + 1) & 1, stg);
        __syncthreads();
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
