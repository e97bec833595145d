// KV append (paper Sec. II-A: the prefill builds the KV cache; Sec. III-C: the
// cache is one pool shared by the prefill and decode sides) and the placement
// probe used to check CU masks.
//
// Append is an index map plus a bit-exact copy: new token i of session s goes
// to logical position P_s + i -> page bt[s][pos / ps], slot pos % ps.
//   K page  [D/8][slot][8] : chunk-major; a token's row is cut into 8-channel chunks
//   V page  [slot/8'][D][8]: transposed in chunks of 8 keys, see v_offset()
// 16 neighbouring lanes hold 16 consecutive tokens of one chunk of D, so each
// store instruction writes runs of neighbouring slots.
// One workgroup of 256 threads takes 16 consecutive rows of the token-major
// input and one KV head.  HBM-bound: 2 * T * 2*Hkv*D*sizeof bytes (read + write).
#include "ag_internal.h"

namespace ag {

namespace {

constexpr int kTok = 16;   // tokens per workgroup

// E is the raw storage element (uint16_t for bf16, uint32_t for fp32).
template <typename E>
struct alignas(16) Chunk8 { E e[8]; };

template <typename E>
__global__ __launch_bounds__(256) void kv_append_kernel(E* __restrict__ k_pool, E* __restrict__ v_pool,
                                                        const E* __restrict__ k_new, const E* __restrict__ v_new,
                                                        const int32_t* __restrict__ bt, int max_pages,
                                                        const int32_t* __restrict__ prefix_lens,
                                                        const int32_t* __restrict__ cu_new, int batch, int total_new,
                                                        int hkv, int d, int ps, int ps_shift)
{
    __shared__ int64_t s_page[kTok];   // physical page of each of the 16 tokens, -1 if past the end
    __shared__ int s_slot[kTok];

    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * kTok;
    const int h = blockIdx.y;

    if (tid < kTok) {
        const int t = t0 + tid;
        int64_t page = -1;
        int slot = 0;
        if (t < total_new) {
            // session s with cu_new[s] <= t < cu_new[s+1]; empty sessions are stepped over
            int lo = 0, hi = batch;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (cu_new[mid] <= t) lo = mid; else hi = mid;
            }
            const int s = lo;
            const int pos = prefix_lens[s] + (t - cu_new[s]);
            page = bt[(int64_t)s * max_pages + (pos >> ps_shift)];
            slot = pos & (ps - 1);
        }
        s_page[tid] = page;
        s_slot[tid] = slot;
    }
    __syncthreads();

    const int chunks = d >> 3;   // 8-element chunks per row
    using C8 = Chunk8<E>;

    // thread (token = tid % 16, chunk = tid / 16 + 16*r): 16 neighbouring lanes hold 16 consecutive
    // tokens of one chunk, so both stores below write runs of neighbouring slots
    const int tok = tid & 15;
    const int64_t page = s_page[tok];
    if (page >= 0) {
        const int slot = s_slot[tok];
        const int64_t row = (int64_t)(t0 + tok) * hkv + h;
        E* kdst = k_pool + ((int64_t)page * hkv + h) * d * ps + (int64_t)slot * 8;        // + chunk * ps * 8
        E* vdst = v_pool + ((int64_t)page * hkv + h) * d * ps;
        for (int c = tid >> 4; c < chunks; c += 16) {
            *reinterpret_cast<C8*>(kdst + (int64_t)c * ps * 8) = *reinterpret_cast<const C8*>(k_new + row * d + c * 8);
            const C8 x = *reinterpret_cast<const C8*>(v_new + row * d + c * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) vdst[v_offset(slot, c * 8 + e, ps, d)] = x.e[e];
        }
    }
}

// Where did this workgroup run?  HW_ID (register 4): CU id bits 8-11, shader
// array bit 12, shader engine bits 13-15; XCC_ID (register 20): bits 0-3.
__global__ __launch_bounds__(64) void probe_kernel(uint32_t* ids, int spin_cycles)
{
    const long long t_end = (long long)clock64() + spin_cycles;
    int guard = 0;
    while ((long long)clock64() < t_end && guard < (1 << 24)) ++guard;   // bounded: always terminates
    if (threadIdx.x == 0) {
        const uint32_t hw = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);
        const uint32_t xcc = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 20);
        const uint32_t cu = (hw >> 8) & 0xF, sa = (hw >> 12) & 0x1, se = (hw >> 13) & 0x7;
        ids[blockIdx.x] = cu | (sa << 8) | (se << 12) | ((xcc & 0xF) << 16);
    }
}

}  // namespace

ag_status launch_kv_append(const CacheView& c, const void* k_new, const void* v_new, const int32_t* bt, int max_pages,
                           const int32_t* prefix_lens, const int32_t* new_lens, const int32_t* cu_new, int batch,
                           int total_new, hipStream_t st)
{
    (void)new_lens;   // cu_new already carries the per-session counts
    const dim3 grid((total_new + kTok - 1) / kTok, c.hkv);
    if (c.dtype == AG_BF16) {
        hipLaunchKernelGGL(kv_append_kernel<uint16_t>, grid, dim3(256), 0, st, (uint16_t*)c.k, (uint16_t*)c.v,
                           (const uint16_t*)k_new, (const uint16_t*)v_new, bt, max_pages, prefix_lens, cu_new, batch,
                           total_new, c.hkv, c.d, c.ps, c.ps_shift);
    } else {
        hipLaunchKernelGGL(kv_append_kernel<uint32_t>, grid, dim3(256), 0, st, (uint32_t*)c.k, (uint32_t*)c.v,
                           (const uint32_t*)k_new, (const uint32_t*)v_new, bt, max_pages, prefix_lens, cu_new, batch,
                           total_new, c.hkv, c.d, c.ps, c.ps_shift);
    }
    return hip_check(hipGetLastError(), "kv_append launch");
}

ag_status launch_probe(uint32_t* ids_out, int n_wg, int spin_cycles, hipStream_t st)
{
    hipLaunchKernelGGL(probe_kernel, dim3(n_wg), dim3(64), 0, st, ids_out, spin_cycles);
    return hip_check(hipGetLastError(), "probe launch");
}

}  // namespace ag
