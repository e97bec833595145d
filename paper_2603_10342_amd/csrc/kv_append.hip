// KV append (paper Sec. II-A: the prefill builds the KV cache; Sec. III-C: the
// cache is one pool shared by the prefill and decode sides) and the placement
// probe used to check CU masks.
//
// Append is an index map plus a bit-exact copy: new token i of session s goes
// to logical position P_s + i -> page bt[s][pos / ps], slot pos % ps.
//   K page  [D/8][slot][8] : chunk-major; a token's row is cut into 8-channel chunks
//   V page  [slot/8'][D][8]: transposed in chunks of 8 keys, see v_offset()
// HBM-bound: 2 * T * 2*Hkv*D*sizeof bytes (read + write).  Two kernels:
//   kv_append_pages_kernel  page size 16: one workgroup per (touched page, KV head), rows staged in LDS
//   kv_append_kernel        any page size: one workgroup of 256 threads takes 16 consecutive rows of the
//                           token-major input and one KV head; 16 neighbouring lanes hold 16 consecutive
//                           tokens of one chunk of D, so each store instruction writes runs of neighbouring slots.
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

// Page-wise append for page size 16 (the fast path).  One workgroup per (touched page of a session, KV head):
// the page's new tokens are read row by row (coalesced) into LDS and written out in the pool layouts with
// 16/32-byte stores: K as runs of neighbouring slots per chunk, V - when the whole page is new, the usual case
// in a prefill - as whole 8-key chunks, 2 KiB contiguous per wave.  A partly filled page (the first and last
// page of an appended range, or a decode step's single token) writes V element by element so that slots that
// already hold older tokens are not touched.
// Items are numbered session-major; a workgroup finds its (session, page) by a wave-wide scan of the
// per-session page counts, 64 sessions at a time.
template <typename E>
__global__ __launch_bounds__(256) void kv_append_pages_kernel(E* __restrict__ k_pool, E* __restrict__ v_pool,
                                                              const E* __restrict__ k_new, const E* __restrict__ v_new,
                                                              const int32_t* __restrict__ bt, int max_pages,
                                                              const int32_t* __restrict__ prefix_lens,
                                                              const int32_t* __restrict__ new_lens,
                                                              const int32_t* __restrict__ cu_new, int batch, int hkv,
                                                              int d)
{
    constexpr int PS = 16;
    using C8 = Chunk8<E>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int s_item[4];            // session, first position, token count, physical page (-1: no such item)
    C8* lds_k = reinterpret_cast<C8*>(smem);                       // [16 tokens][d/8]
    C8* lds_v = lds_k + PS * (d >> 3);

    const int tid = threadIdx.x, lane = tid & 63;
    const int item = blockIdx.x, h = blockIdx.y;
    const int chunks = d >> 3;

    if (tid < 64) {
        int acc = 0, found = -1, first_pos = 0, count = 0;
        for (int base = 0; base < batch && found < 0; base += 64) {
            const int s = base + lane;
            int p = 0, n = 0;
            if (s < batch) { p = prefix_lens[s]; n = new_lens[s]; }
            const int np = n > 0 ? ((p + n - 1) >> 4) - (p >> 4) + 1 : 0;
            int scan = np;                                           // inclusive scan over the 64 lanes
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int up = __shfl_up(scan, o);
                if (lane >= o) scan += up;
            }
            const uint64_t hit = __builtin_amdgcn_ballot_w64(acc + scan > item);
            if (hit) {
                const int l = __builtin_ctzll(hit);                  // first session whose pages reach the item
                const int before = acc + __shfl(scan, l) - __shfl(np, l);
                const int pl = __shfl(p, l), nl = __shfl(n, l);
                const int lp = (pl >> 4) + (item - before);
                found = base + l;
                first_pos = max(pl, lp << 4);
                count = min(pl + nl, (lp + 1) << 4) - first_pos;
            }
            acc += __shfl(scan, 63);
        }
        if (lane == 0) {
            s_item[0] = found;
            s_item[1] = first_pos;
            s_item[2] = count;
            s_item[3] = found >= 0 ? bt[(int64_t)found * max_pages + (first_pos >> 4)] : -1;
        }
    }
    __syncthreads();
    const int s = s_item[0];
    if (s < 0) return;                                               // beyond the last touched page
    const int pos0 = s_item[1], n_tok = s_item[2];
    const int64_t page = s_item[3];
    const int slot0 = pos0 & (PS - 1);
    const int64_t t0 = (int64_t)cu_new[s] + (pos0 - prefix_lens[s]);

    for (int idx = tid; idx < n_tok * chunks; idx += 256) {          // rows in, 16 lanes per 8-chunk run
        const int row = idx / chunks, c = idx - row * chunks;
        const int64_t src = ((t0 + row) * hkv + h) * d + c * 8;
        lds_k[idx] = *reinterpret_cast<const C8*>(k_new + src);
        lds_v[idx] = *reinterpret_cast<const C8*>(v_new + src);
    }
    __syncthreads();

    E* kpage = k_pool + (page * hkv + h) * (int64_t)d * PS;
    E* vpage = v_pool + (page * hkv + h) * (int64_t)d * PS;
    for (int idx = tid; idx < n_tok * chunks; idx += 256) {          // K: neighbouring lanes, neighbouring slots
        const int c = idx / n_tok, i = idx - c * n_tok;
        *reinterpret_cast<C8*>(kpage + ((int64_t)c * PS + slot0 + i) * 8) = lds_k[i * chunks + c];
    }
    const E* lv = reinterpret_cast<const E*>(lds_v);                 // [token][d]
    if (n_tok == PS) {                                               // whole page: V as 8-key chunks
        for (int idx = tid; idx < 2 * d; idx += 256) {
            const int half = idx / d, ch = idx - half * d;
            C8 x;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x.e[e] = lv[(half * 4 + e) * d + ch];
                x.e[4 + e] = lv[(8 + half * 4 + e) * d + ch];
            }
            *reinterpret_cast<C8*>(vpage + ((int64_t)half * d + ch) * 8) = x;
        }
    } else {
        for (int idx = tid; idx < n_tok * d; idx += 256) {
            const int ch = idx / n_tok, i = idx - ch * n_tok;
            vpage[v_offset(slot0 + i, ch, PS, d)] = lv[i * d + ch];
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
    if (c.ps == 16) {
        // every session touches at most N_s / 16 + 2 pages: total_new / 16 + 2 * batch items bound the launch
        const int64_t items = total_new / 16 + 2 * (int64_t)batch;
        if (items > 0x7fffffff || c.hkv > 65535) { set_error("append too large for one launch"); return AG_ERR_INVALID_ARG; }
        const dim3 grid((unsigned)items, c.hkv);
        const size_t lds = 2 * 16 * (size_t)c.d * (c.dtype == AG_BF16 ? 2 : 4);
        if (c.dtype == AG_BF16)
            hipLaunchKernelGGL(kv_append_pages_kernel<uint16_t>, grid, dim3(256), lds, st, (uint16_t*)c.k, (uint16_t*)c.v,
                               (const uint16_t*)k_new, (const uint16_t*)v_new, bt, max_pages, prefix_lens, new_lens,
                               cu_new, batch, c.hkv, c.d);
        else
            hipLaunchKernelGGL(kv_append_pages_kernel<uint32_t>, grid, dim3(256), lds, st, (uint32_t*)c.k, (uint32_t*)c.v,
                               (const uint32_t*)k_new, (const uint32_t*)v_new, bt, max_pages, prefix_lens, new_lens,
                               cu_new, batch, c.hkv, c.d);
        return hip_check(hipGetLastError(), "kv_append launch");
    }
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
