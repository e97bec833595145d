// Pieces shared by the two split-K kernels over a paged KV cache (bf16, head_dim 128, page 16): the decode
// step and the merged decode + short-resume batch.  Internal; nothing here is part of the ABI.
#pragma once

#include "ag_internal.h"

namespace ag {
namespace splitk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int PS = 16;

// Tokens of one part of a session's context when it is cut for splits of at most `split` tokens:
// n = ceil(ctx / split) equal parts, each a multiple of 128 (32 per wave step x 4 waves).
__host__ __device__ inline int part_tokens(int ctx, int split)
{
    const int n = (ctx + split - 1) / split;
    return (((ctx + n - 1) / n) + 127) & ~127;
}
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ bf16x8 ld16(const __bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }
// The same load with the streaming hint: K and V are read once per step and never again by this launch, and
// loads marked non-temporal measure 10-15 % more HBM bandwidth on this chip than plain ones.
__device__ __forceinline__ bf16x8 ld16_stream(const __bf16* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(p));
}

// v holds 8 tokens: elements 0..3 are tokens j = 0..3, elements 4..7 tokens j = 8..11 of the lane's run.
// Zero element e < 4 unless e < keep_lo, and element 4 + e unless e < keep_hi.
__device__ __forceinline__ bf16x8 keep_quads(bf16x8 v, int keep_lo, int keep_hi)
{
    u32x4 u = __builtin_bit_cast(u32x4, v);
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        u[w] &= ((2 * w < keep_lo) ? 0x0000FFFFu : 0u) | ((2 * w + 1 < keep_lo) ? 0xFFFF0000u : 0u);
        u[2 + w] &= ((2 * w < keep_hi) ? 0x0000FFFFu : 0u) | ((2 * w + 1 < keep_hi) ? 0xFFFF0000u : 0u);
    }
    return __builtin_bit_cast(bf16x8, u);
}

struct StepRegs {       // one wave's K and V operands for 32 tokens (two pages)
    bf16x8 k1[4], k2[4], v[8];
};


// The partials (m, l, O[D]) of one (row, head) lie at slots base .. base + n - 1 (n >= 1, the first of them with a
// finite m); combine them in slot order - reproducible - four at a time, so that a group's loads are in flight
// together instead of one dependent round trip per partial.  Returns channel d of the normalised output.
// kCoherent: the partials were written by other workgroups of the SAME launch (device-scope stores, see
// store_coherent): read them with device-scope loads, which do not hit in this XCD's caches.
__device__ __forceinline__ float load_coherent(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void store_coherent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

template <bool kCoherent = false>
__device__ __forceinline__ float merge_partials(const float* __restrict__ ws_o, const float* __restrict__ ws_ml,
                                                int64_t base, int n, int d)
{
    float ms = -INFINITY, acc = 0.f, l = 0.f;
    for (int i0 = 0; i0 < n; i0 += 4) {
        float mi[4], li[4], oi[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t p = base + min(i0 + j, n - 1);
            mi[j] = kCoherent ? load_coherent(ws_ml + p * 2) : ws_ml[p * 2];
            li[j] = kCoherent ? load_coherent(ws_ml + p * 2 + 1) : ws_ml[p * 2 + 1];
            oi[j] = kCoherent ? load_coherent(ws_o + p * D + d) : ws_o[p * D + d];
            if (i0 + j >= n) mi[j] = -INFINITY;
        }
        const float m_new = fmaxf(fmaxf(ms, fmaxf(mi[0], mi[1])), fmaxf(mi[2], mi[3]));
        const float keep = ms == -INFINITY ? 0.f : exp2f(ms - m_new);
        acc *= keep;
        l *= keep;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float f = mi[j] == -INFINITY ? 0.f : exp2f(mi[j] - m_new);     // a partial that saw no key
            acc += f * oi[j];
            l += f * li[j];
        }
        ms = m_new;
    }
    return acc / l;
}

// Workspace is sized for the smallest split a launcher may choose.
constexpr int kMinSplit = 256;
inline int splits_for(int max_ctx, int split) { return max_ctx <= 0 ? 1 : (max_ctx + split - 1) / split; }

}  // namespace splitk
}  // namespace ag
