// General paged softmax attention in fp32 arithmetic: any supported head_dim,
// page size and storage dtype, for all three request classes (paper Sec. I,
// Sec. II-A): row i of session s sits at position P_s + i and sees keys
// 0 .. P_s + i; a decode step is the one-row case at position ctx_len - 1.
//
// One wavefront per (row, query head).  Keys are taken 64 at a time, one per
// lane (score = scale * q.k in fp32, then a streaming softmax: running max m,
// running sum l, accumulator rescaled when m grows); values are accumulated
// with lane = channel.  It is the path for fp32 caches and for shapes the
// matrix-core kernels do not cover; it is not tuned for bandwidth.
#include "ag_internal.h"

namespace ag {

namespace {

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__bf16 x) { return (float)x; }
__device__ __forceinline__ void store_out(float* p, float x) { *p = x; }
__device__ __forceinline__ void store_out(__bf16* p, float x) { *p = (__bf16)x; }   // round to nearest even

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_general_kernel(AttnArgs a)
{
    __shared__ float s_q[4][256];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + w;
    if (item >= (int64_t)a.total_rows * a.hq) return;   // whole wave leaves; no block barrier is used below
    const int t = (int)(item / a.hq), h = (int)(item % a.hq);
    const int D = a.c.d, ps = a.c.ps, hkv = a.c.hkv;
    const int g = h / (a.hq / hkv);

    int s, pos;
    if (a.cu_new == nullptr) {           // decode: one row per session
        s = t;
        pos = a.ctx_lens[s] - 1;
    } else {
        int lo = 0, hi = a.batch;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (a.cu_new[mid] <= t) lo = mid; else hi = mid;
        }
        s = lo;
        pos = (a.prefix_lens ? a.prefix_lens[s] : 0) + (t - a.cu_new[s]);
    }
    T* out = (T*)a.out + ((int64_t)t * a.hq + h) * D;
    if (pos < 0) {                        // empty context: defined as a row of zeros
        for (int d = lane; d < D; d += 64) store_out(out + d, 0.0f);
        return;
    }

    const T* q = (const T*)a.q + ((int64_t)t * a.hq + h) * D;
    for (int d = lane; d < D; d += 64) s_q[w][d] = to_f32(q[d]);
    __builtin_amdgcn_wave_barrier();      // s_q[w] is private to this wave

    const T* kp = (const T*)a.c.k;
    const T* vp = (const T*)a.c.v;
    const int32_t* bt = a.bt + (int64_t)s * a.max_pages;

    float m = -INFINITY, l = 0.0f;
    float o[4] = {0.0f, 0.0f, 0.0f, 0.0f};   // channels lane, lane+64, lane+128, lane+192

    for (int base = 0; base <= pos; base += 64) {
        const int j = base + lane;
        const bool valid = j <= pos;
        int64_t page = 0;
        int slot = 0;
        float x = -INFINITY;
        if (valid) {
            page = bt[j >> a.c.ps_shift];
            slot = j & (ps - 1);
            const T* kr = kp + (page * hkv + g) * (int64_t)D * ps + slot * 8;   // chunk c of this slot: + c * ps * 8
            float dot = 0.0f;
            for (int d = 0; d < D; ++d) dot = fmaf(s_q[w][d], to_f32(kr[(int64_t)(d >> 3) * ps * 8 + (d & 7)]), dot);
            x = a.scale * dot;
        }
        const float m_new = fmaxf(m, wave_max(x));      // finite: lane 0 of every block is valid
        const float alpha = expf(m - m_new);            // exp(-inf) = 0 on the first block
        const float p = valid ? expf(x - m_new) : 0.0f;
        l = l * alpha + wave_sum(p);
#pragma unroll
        for (int c = 0; c < 4; ++c) o[c] *= alpha;
        const int cnt = min(64, pos - base + 1);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj);
            const int64_t pg = __shfl((int)page, jj);
            const int sl = __shfl(slot, jj);
            const T* vr = vp + (pg * hkv + g) * (int64_t)D * ps;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int d = lane + 64 * c;
                if (d < D) o[c] = fmaf(pj, to_f32(vr[v_offset(sl, d, ps, D)]), o[c]);
            }
        }
        m = m_new;
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int d = lane + 64 * c;
        if (d < D) store_out(out + d, o[c] * inv);
    }
}

}  // namespace

ag_status launch_attn_general(const AttnArgs& a, hipStream_t st)
{
    const int64_t items = (int64_t)a.total_rows * a.hq;
    const int64_t blocks = (items + 3) / 4;
    if (blocks > 0x7fffffff) { set_error("too many rows for one launch"); return AG_ERR_INVALID_ARG; }
    prof_before(st);
    if (a.c.dtype == AG_BF16)
        hipLaunchKernelGGL(attn_general_kernel<__bf16>, dim3((unsigned)blocks), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(attn_general_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, a);
    prof_after(st);
    return hip_check(hipGetLastError(), "attn_general launch");
}

}  // namespace ag
