// The 64-key x 32-query tile arithmetic of the matrix-core attention kernels (bf16, head_dim 128, page 16):
// S^T = K . Q^T and O^T += V^T . P^T on 32x32x16 MFMA with K and V tiles in LDS, and the softmax weights of a
// tile under a reference maximum.  Shared by the prefill kernel and by the rows items of the merged decode-queue
// kernel, which walk the same tiles over a part of the keys.  Internal; nothing here is part of the ABI.
#pragma once

#include "ag_internal.h"

namespace ag {
namespace tile32 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int PS = 16;
constexpr int BN = 64;                  // keys per tile
// LDS tiles are chunk-major, like the pages themselves, and are filled by direct global-to-LDS loads:
//   K tile [chunk c = 0..15][key 0..63][8 ch]   operand of key n, chunk c at (c * 64 + n) * 16 bytes
//   V tile [chunk q = 0..7 ][ch  0..127][8 keys] operand of channel d, chunk q at (q * 128 + d) * 16 bytes
// (q = 2 * page + half; the 8 keys of a chunk are slots half*4 + {0..3} and 8 + half*4 + {0..3} of the page).
// The 32 lanes of a half-wave read 32 consecutive 16-byte pieces: conflict free, and every operand address
// is the lane's base plus a compile-time offset.
constexpr int kTile = BN * D * 2;       // 16 KiB, K and V alike
constexpr int kKStages = 3;             // K(t+2) is requested while K(t) is used
constexpr float kRescaleSlack = 8.0f;   // log2 units a row's maximum may exceed m when the ordered path leaves m alone
constexpr float kWeightSumLimit = 16384.0f;   // a lane's 32 weights of a tile may sum to this much before m is moved
constexpr float kLog2e = 1.4426950408889634f;

constexpr int kOperandsAhead = 3;       // LDS operand reads run this many matrix instructions ahead of their use

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

// S^T tile (64 keys x 32 queries) = K tile . Q^T.  kb: this lane's base in a K tile (key n, chunk hi).
// Operand reads run kAhead matrix instructions ahead of their use; the two key blocks alternate so that
// neighbouring matrix instructions write different accumulators.
__device__ __forceinline__ void qk_tile(const unsigned char* kb, const bf16x8 (&qf)[8], f32x16 (&sc)[2])
{
    constexpr int kAhead = kOperandsAhead;
    bf16x8 opnd[kAhead + 1];
    auto operand = [&](int i) -> const unsigned char* { return kb + (i & 1) * 512 + (i >> 1) * 2048; };   // (ks, b)
#pragma unroll
    for (int i = 0; i < kAhead; ++i) opnd[i] = *reinterpret_cast<const bf16x8*>(operand(i));
    // the first matrix instruction of each key block starts from a literal zero: no accumulator to clear
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (i + kAhead < 16) opnd[(i + kAhead) % (kAhead + 1)] = *reinterpret_cast<const bf16x8*>(operand(i + kAhead));
        sc[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i % (kAhead + 1)], qf[i >> 1], i < 2 ? zero : sc[i & 1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// O^T (128 channels x 32 queries) += V^T tile . P^T.  vb: this lane's base in a V tile (channel n, chunk hi).
// Same operand ring as qk_tile (it also bounds the registers the compiler may spend on early reads).
__device__ __forceinline__ void pv_tile(const unsigned char* vb, const bf16x8 (&pb)[4], f32x16 (&o)[4])
{
    constexpr int kAhead = kOperandsAhead;
    bf16x8 opnd[kAhead + 1];
    auto operand = [&](int i) -> const unsigned char* { return vb + (i & 3) * 512 + (i >> 2) * 4096; };   // (j, mb)
#pragma unroll
    for (int i = 0; i < kAhead; ++i) opnd[i] = *reinterpret_cast<const bf16x8*>(operand(i));
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (i + kAhead < 16) opnd[(i + kAhead) % (kAhead + 1)] = *reinterpret_cast<const bf16x8*>(operand(i + kAhead));
        o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i % (kAhead + 1)], pb[i >> 2], o[i & 3], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
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

// P^T = exp2(S^T * sl2 - m) packed as the B operands of the four k-steps of the second product; adds to lsum
// the weights as rounded to bf16 (what the value product multiplies by), one dot2 per packed pair.
__device__ __forceinline__ void exp_tile(const f32x16 (&sc)[2], float sl2, float m, float& lsum, bf16x8 (&pb)[4])
{
    const bf16x2 kOnes = {(__bf16)1.0f, (__bf16)1.0f};
    float psum = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            const bf16x2 pr = {(__bf16)__builtin_amdgcn_exp2f(fmaf(sc[b][i], sl2, -m)),
                               (__bf16)__builtin_amdgcn_exp2f(fmaf(sc[b][i + 1], sl2, -m))};
            psum = __builtin_amdgcn_fdot2_f32_bf16(pr, kOnes, psum, false);
            pb[b * 2 + (i >> 3)][i & 7] = pr[0];
            pb[b * 2 + (i >> 3)][(i & 7) + 1] = pr[1];
        }
    lsum += psum;
}

// One iteration's vector work and second product for a wave: P(t) = exp2(S(t) - m) into p_cur (if do_sm) side
// by side with O += V(t-1) . P(t-1) from p_prev (if do_pv); vb is the lane's base in the V(t-1) tile.
// m is a reference, not the running maximum, and the common case does not even look for the tile's maximum:
// it takes the weights under the current m and checks afterwards that none came out large (a lane's sum of 32
// weights at most 2^14, so no weight above 2^14; inf and NaN fail the test too - a query that has not seen a
// key yet has m = -inf).  Only then, and on a wave's first tile, the ordered path finds the row maxima and
// moves m.
__device__ __forceinline__ void softmax_and_value_product(bool do_sm, bool do_pv, const unsigned char* vb,
                                                          const f32x16 (&sc)[2], float sl2, float& m, float& lsum,
                                                          const bf16x8 (&p_prev)[4], bf16x8 (&p_cur)[4], f32x16 (&o)[4])
{
    bool redo = false;
    if (do_sm && do_pv) {
        // the common case: two independent pieces, interleaved by hand.  Step i issues the operand read
        // of matrix instruction i + kAhead, matrix instruction i, and the exp of scores 2i and 2i + 1;
        // the fences keep the compiler from regrouping them.  Neighbouring matrix instructions belong
        // to different accumulators.
        constexpr int kAhead = kOperandsAhead;
        bf16x8 opnd[kAhead + 1];
        auto operand = [&](int i) -> const unsigned char* {   // order (j, mb)
            return vb + (i & 3) * 512 + (i >> 2) * 4096;
        };
#pragma unroll
        for (int i = 0; i < kAhead; ++i) opnd[i] = *reinterpret_cast<const bf16x8*>(operand(i));
        const bf16x2 kOnes = {(__bf16)1.0f, (__bf16)1.0f};
        float psum = 0.f;
        // The vector work of a pair of scores is a chain (scale -> exp -> convert -> sum) whose links cannot
        // issue back to back; it is spread over four steps so that nothing inside a step depends on anything
        // else inside it: step i scales pair i + 1, takes the exp of pair i, converts pair i - 1 and sums
        // pair i - 2.
        auto scaled = [&](int pair, int k) { const int e = 2 * pair + k; return fmaf(sc[e >> 4][e & 15], sl2, -m); };
        float x0 = scaled(0, 0), x1 = scaled(0, 1);          // pair 0, scaled
        float q0 = 0.f, q1 = 0.f;                            // exp of the pair one step back
        bf16x2 pr_prev = {(__bf16)0.f, (__bf16)0.f};         // converted pair two steps back
#pragma unroll
        for (int i = 0; i < 16 + 2; ++i) {
            if (i < 16) {
                if (i + kAhead < 16) opnd[(i + kAhead) % (kAhead + 1)] = *reinterpret_cast<const bf16x8*>(operand(i + kAhead));
                o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i % (kAhead + 1)], p_prev[i >> 2], o[i & 3], 0, 0, 0);
            }
            if (i >= 2) psum = __builtin_amdgcn_fdot2_f32_bf16(pr_prev, kOnes, psum, false);   // l sums the weights as rounded
            if (i >= 1 && i <= 16) {
                const bf16x2 pr = {(__bf16)q0, (__bf16)q1};
                const int e = 2 * (i - 1);
                p_cur[e >> 3][e & 7] = pr[0];
                p_cur[e >> 3][(e & 7) + 1] = pr[1];
                pr_prev = pr;
            }
            if (i < 16) {
                q0 = __builtin_amdgcn_exp2f(x0);
                q1 = __builtin_amdgcn_exp2f(x1);
            }
            if (i + 1 < 16) { x0 = scaled(i + 1, 0); x1 = scaled(i + 1, 1); }
            __builtin_amdgcn_sched_barrier(0);
        }
        redo = __builtin_amdgcn_ballot_w64(!(psum <= kWeightSumLimit)) != 0;      // uniform over the wave
        if (!redo) lsum += psum;
    }
    if (!(do_sm && do_pv) || redo) {
        if (do_pv && !redo) pv_tile(vb, p_prev, o);      // (a redo has done the value product already)
        if (do_sm) {
            float mx = row_max(sc) * sl2;            // scale > 0: max and scaling commute
            // m is shared by the two lanes of a query: if either lane's own maximum outgrew m, combine them
            if (__builtin_amdgcn_ballot_w64(mx > m + kRescaleSlack) != 0) {
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m, mx);
                // (a query that still has seen no key has m = m_new = -inf: nothing to rescale)
                const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m - m_new);
                lsum *= alpha;
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[mb][i] *= alpha;
                m = m_new;
            }
            // a query that has seen no key yet (none of a part's keys so far lies at or below its position)
            // keeps m = -inf: its scores are all -inf as well, and the weights must come out 0, not NaN
            exp_tile(sc, sl2, m == -INFINITY ? 0.f : m, lsum, p_cur);
        }
    }
}

}  // namespace tile32
}  // namespace ag
