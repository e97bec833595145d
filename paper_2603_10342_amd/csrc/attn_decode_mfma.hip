// Short GQA decode over a paged KV cache, bf16, head_dim 128, page 16
// (paper Sec. II-A: decode reuses the cached keys and values, linear in the
// context; Sec. III-B: one token per active stream per decode step).
//
// The step is bound by HBM: every cached K and V byte is read once
// (2 * Hkv * 128 * 2 B = 4 KiB per token at 8 KV heads) and the arithmetic is
// Hq / Hkv flop per byte.  All G = Hq / Hkv query heads that share a KV head
// are processed together so each byte is fetched once, and the two small
// contractions run on the matrix cores so that the vector ALUs only do the
// softmax bookkeeping:
//
//   split kernel, one workgroup (4 waves) per (session, KV head, 512-token split);
//   each wave owns 128 consecutive tokens and walks them 32 (two pages) at a time:
//     S^T[token][head] = K[token][:] . Q[head][:]     2 x 4 MFMA 16x16x32 (heads padded to 16)
//     streaming softmax on S^T (running max m, running sum l; exp2 with log2(e) folded in)
//     O^T[d][head]    += V^T[d][token] . P^T[token][head]   8 MFMA 16x16x32
//   K rows are loaded straight into the A-operand layout (lane = token row,
//   16 B = 8 channels); V pages are stored transposed ([d][slot]) so a lane's
//   16 B load is 8 consecutive tokens of one channel, which is the A operand
//   of the second product.  The MFMA row order of the first product is
//   chosen so that the 8 scores a lane ends up with are exactly the 8
//   tokens its V load covers: no cross-lane shuffles between the products.
//   The 4 waves are merged in LDS and the workgroup writes one partial
//   (m, l, O) per query head to the workspace;
//
//   merge kernel, one workgroup per (session, query head): combines the
//   partials of all splits in split order (reproducible) and writes bf16.
#include "ag_internal.h"

namespace ag {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int PS = 16;
constexpr int kWaveTok = kDecodeSplit / 4;   // 128 tokens per wave
constexpr int kSteps = kWaveTok / 32;        // two pages per step
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ bf16x8 ld16(const __bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }

// zero the elements e of a packed bf16x8 whose index is >= keep (0 <= keep < 8 on entry means partial)
__device__ __forceinline__ bf16x8 keep_first(bf16x8 v, int keep)
{
    u32x4 u = __builtin_bit_cast(u32x4, v);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t lo = (2 * w < keep) ? 0x0000FFFFu : 0u;
        const uint32_t hi = (2 * w + 1 < keep) ? 0xFFFF0000u : 0u;
        u[w] &= (lo | hi);
    }
    return __builtin_bit_cast(bf16x8, u);
}

__global__ __launch_bounds__(256, 2) void decode_split_kernel(AttnArgs a, float* __restrict__ ws_o,
                                                              float* __restrict__ ws_ml, int n_splits_max)
{
    __shared__ float s_o[4][16][D];     // per wave, per (padded) head: unnormalised O
    __shared__ float s_m[4][16];
    __shared__ float s_l[4][16];

    const int split = blockIdx.x, g = blockIdx.y, s = blockIdx.z;
    const int ctx = a.ctx_lens[s];
    const int start = split * kDecodeSplit;
    if (start >= ctx) return;            // uniform over the workgroup; covers ctx == 0

    const int hkv = a.c.hkv, hq = a.hq;
    const int G = hq / hkv;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, c = lane >> 4;
    const int wstart = start + w * kWaveTok;

    const __bf16* kpool = (const __bf16*)a.c.k;
    const __bf16* vpool = (const __bf16*)a.c.v;

    // Q^T as the B operand: column = head r (zero beyond G), k = channels kk*32 + c*8 .. +7
    bf16x8 qf[4];
    {
        const __bf16* qrow = (const __bf16*)a.q + ((int64_t)s * hq + (int64_t)g * G + (r < G ? r : 0)) * D + c * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 x = ld16(qrow + kk * 32);
            if (r >= G) x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qf[kk] = x;
        }
    }

    // physical pages of this wave's 8 logical pages (clamped to the session's last page)
    const int n_pages_ctx = (ctx + PS - 1) >> 4;
    int my_pid;
    {
        const int lp = min((wstart >> 4) + (lane & 7), n_pages_ctx - 1);
        my_pid = a.bt[(int64_t)s * a.max_pages + lp];
    }

    const float sl2 = a.scale * kLog2e;
    float m = -INFINITY, lsum = 0.0f;
    f32x4 o[8];
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // row r of the first product: page (r >> 3), slot ((r >> 2) & 1) * 8 + (r & 3); second product: slot + 4
    const int k_pg = r >> 3;
    const int k_slot = ((r >> 2) & 1) * 8 + (r & 3);
    const int v_pg = c >> 1;
    const int v_slot = (c & 1) * 8;

#pragma unroll 1
    for (int st = 0; st < kSteps; ++st) {
        const int tok0 = wstart + st * 32;
        if (tok0 >= ctx) break;          // uniform over the wave
        const int64_t pA = __builtin_amdgcn_readlane(my_pid, 2 * st);
        const int64_t pB = __builtin_amdgcn_readlane(my_pid, 2 * st + 1);

        const __bf16* kp = kpool + ((((k_pg ? pB : pA) * hkv + g) * PS + k_slot) * D) + c * 8;
        const __bf16* vp = vpool + ((((v_pg ? pB : pA) * hkv + g) * D + r) * PS) + v_slot;
        bf16x8 k1[4], k2[4], v[8];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            k1[kk] = ld16(kp + kk * 32);
            k2[kk] = ld16(kp + 4 * D + kk * 32);
        }
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) v[mb] = ld16(vp + mb * 16 * PS);

        f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1[kk], qf[kk], s1, 0, 0, 0);
            s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k2[kk], qf[kk], s2, 0, 0, 0);
        }
        // this lane's 8 scores are tokens tokb .. tokb + 7 of head r (s1: +0..3, s2: +4..7)
        const int tokb = tok0 + c * 8;
        const int keep = ctx - tokb;     // tokens tokb + e with e < keep exist
        float x[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[i] = (i < keep) ? s1[i] * sl2 : -INFINITY;
            x[4 + i] = (4 + i < keep) ? s2[i] * sl2 : -INFINITY;
        }
        float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m, mx);          // finite: token tok0 exists
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        float psum = 0.f;
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float p = __builtin_amdgcn_exp2f(x[e] - m_new);
            psum += p;
            pb[e] = (__bf16)p;
        }
        lsum = lsum * alpha + psum;
        m = m_new;
        if (tok0 + 32 > ctx) {           // last, partial step: unwritten slots may hold anything, NaN included
            const int kp8 = keep < 0 ? 0 : keep;
#pragma unroll
            for (int mb = 0; mb < 8; ++mb) v[mb] = keep_first(v[mb], kp8);
        }
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) {
            o[mb] *= alpha;
            o[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v[mb], pb, o[mb], 0, 0, 0);
        }
    }
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);

    // o[mb][i] is O^T[d = mb*16 + c*4 + i][head r]
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) *reinterpret_cast<f32x4*>(&s_o[w][r][mb * 16 + c * 4]) = o[mb];
    if (c == 0) { s_m[w][r] = m; s_l[w][r] = lsum; }
    __syncthreads();

    for (int idx = threadIdx.x; idx < G * D; idx += 256) {
        const int head = idx >> 7, d = idx & (D - 1);
        float ms = s_m[0][head];
#pragma unroll
        for (int ww = 1; ww < 4; ++ww) ms = fmaxf(ms, s_m[ww][head]);
        float acc = 0.f, l = 0.f;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) {
            const float f = exp2f(s_m[ww][head] - ms);   // a wave without tokens has m = -inf -> 0
            acc += f * s_o[ww][head][d];
            l += f * s_l[ww][head];
        }
        const int64_t slot = ((int64_t)s * hq + (int64_t)g * G + head) * n_splits_max + split;
        ws_o[slot * D + d] = acc;
        if (d == 0) { ws_ml[slot * 2] = ms; ws_ml[slot * 2 + 1] = l; }
    }
}

__global__ __launch_bounds__(128) void decode_merge_kernel(AttnArgs a, const float* __restrict__ ws_o,
                                                           const float* __restrict__ ws_ml, int n_splits_max)
{
    const int row = blockIdx.x;                 // s * hq + h
    const int s = row / a.hq;
    const int d = threadIdx.x;
    const int ctx = a.ctx_lens[s];
    __bf16* out = (__bf16*)a.out + (int64_t)row * D;
    if (ctx <= 0) { out[d] = (__bf16)0.0f; return; }
    const int n = (ctx + kDecodeSplit - 1) / kDecodeSplit;
    const int64_t base = (int64_t)row * n_splits_max;
    float ms = -INFINITY;
    for (int i = 0; i < n; ++i) ms = fmaxf(ms, ws_ml[(base + i) * 2]);
    float acc = 0.f, l = 0.f;
    for (int i = 0; i < n; ++i) {               // fixed order: reproducible
        const float f = exp2f(ws_ml[(base + i) * 2] - ms);
        acc += f * ws_o[(base + i) * D + d];
        l += f * ws_ml[(base + i) * 2 + 1];
    }
    out[d] = (__bf16)(acc / l);
}

inline int splits_for(int max_ctx) { return max_ctx <= 0 ? 1 : (max_ctx + kDecodeSplit - 1) / kDecodeSplit; }

}  // namespace

size_t decode_workspace_bytes(int batch, int hq, int d, int max_ctx)
{
    return (size_t)batch * hq * splits_for(max_ctx) * (size_t)(d + 2) * sizeof(float);
}

bool decode_mfma_supported(const AttnArgs& a)
{
    return a.c.dtype == AG_BF16 && a.c.d == D && a.c.ps == PS && (a.hq / a.c.hkv) <= 16 &&
           (((uintptr_t)a.q | (uintptr_t)a.c.k | (uintptr_t)a.c.v) % 16 == 0);
}

ag_status launch_decode_mfma(const AttnArgs& a, void* ws, hipStream_t st)
{
    const int nsm = splits_for(a.max_ctx);
    float* ws_o = (float*)ws;
    float* ws_ml = ws_o + (size_t)a.batch * a.hq * nsm * D;
    if (a.batch > 65535 || a.c.hkv > 65535) { set_error("batch or KV heads beyond one launch grid"); return AG_ERR_INVALID_ARG; }
    if (a.max_ctx > 0) {
        prof_before(st);
        hipLaunchKernelGGL(decode_split_kernel, dim3(nsm, a.c.hkv, a.batch), dim3(256), 0, st, a, ws_o, ws_ml, nsm);
        prof_after(st);
        ag_status e = hip_check(hipGetLastError(), "decode split launch");
        if (e) return e;
    }
    hipLaunchKernelGGL(decode_merge_kernel, dim3(a.batch * a.hq), dim3(128), 0, st, a, ws_o, ws_ml, nsm);
    return hip_check(hipGetLastError(), "decode merge launch");
}

}  // namespace ag
