// Short GQA decode over a paged KV cache, bf16, head_dim 128, page 16
// (paper Sec. II-A: decode reuses the cached keys and values, linear in the
// context; Sec. III-B: one token per active stream per decode step).
//
// The step is bound by HBM: every cached K and V byte is read once
// (2 * Hkv * 128 * 2 B = 4 KiB per token at 8 KV heads) and the arithmetic is
// Hq / Hkv flop per byte.  All G = Hq / Hkv query heads that share a KV head
// are processed together so each byte is fetched once, and the two small
// contractions run on the matrix cores so that the vector ALUs only do the
// softmax bookkeeping.
//
// Work is dealt in equal shares.  The memory system serves the CUs at about equal rates while all of them
// stream, so a launch ends when the CU with the most bytes ends: with one workgroup per (session, head, part of
// the context) the CUs that drew long parts ran up to 45 % over the mean and the step took 112 us where the
// bytes need 95.  Instead, the (session, KV head) pairs are laid end to end in units of one wave step
// (32 tokens, two pages), F steps in all, and workgroup w of W takes steps [w q, (w + 1) q) with
// q = max(8, ceil(F / W)): every workgroup, hence every CU, moves the same number of bytes.  A workgroup's
// share covers one pair or the end of one and the start of the next (a "segment" each); every workgroup
// derives the plan itself from the context lengths (a sum and a scan over the batch: the lengths live on
// the device, and a planning launch ahead of this one would cost more than it saves).
//
//   split kernel, per segment: the 4 waves take contiguous quarters and walk them one step at a time:
//     S^T[token][head] = K[token][:] . Q[head][:]     2 x 4 MFMA 16x16x32 (heads padded to 16)
//     streaming softmax on S^T (running max m, running sum l; exp2 with log2(e) folded in)
//     O^T[d][head]    += V^T[d][token] . P^T[token][head]   8 MFMA 16x16x32
//   K rows are loaded straight into the A-operand layout (lane = token row,
//   16 B = 8 channels; pages are chunk-major so 8 neighbouring lanes read 128
//   contiguous bytes); V pages are stored transposed in chunks of 8 keys, so a
//   lane's 16 B load is 8 tokens of one channel, the A operand of the second
//   product.  The MFMA row order of the first product is chosen so that the
//   8 scores a lane ends up with are exactly the 8 tokens its V load covers:
//   no cross-lane shuffles between the products.
//   The 4 waves are merged in LDS and the workgroup writes one partial
//   (m, l, O) per query head and segment to the workspace;
//
//   merge kernel, one workgroup per (session, query head): combines the
//   partials of the pair's segments in order (reproducible) and writes bf16.
#include <algorithm>
#include <atomic>
#include <mutex>

#include "attn_split_common.h"

// Workspace of ag_attn_decode_static: the decode step's header and partials for callers that cannot hand over
// device memory of their own.  One copy per GPU the library runs on, held until the process ends.  In host code
// the name below is only a handle for hipGetSymbolAddress; kernels and copies get the address that call returns.
static __device__ __align__(256) unsigned char scratch[AG_DECODE_STATIC_SCRATCH_BYTES];

namespace ag {

namespace {

using namespace splitk;

constexpr int kMinSteps = kMinSplit / 32;      // a workgroup's share is at least this many steps (256 tokens)
constexpr int kMaxSteps = 128;                 // and at most this many (the launcher sizes the grid for it)

__device__ __forceinline__ int steps_of(int ctx) { return ctx > 0 ? (ctx + 31) >> 5 : 0; }

// Segments a pair of n steps starting at flat step a may be cut into when shares are q >= kMinSteps steps.
inline int pieces_max(int max_ctx) { return (((max_ctx + 31) / 32) - 1) / kMinSteps + 2; }
// Workspace: header [q, then the exclusive step count before each session], partials O, partials (m, l).
inline size_t header_ints(int batch) { return ((size_t)batch + 1 + 3) & ~(size_t)3; }

// What the whole-step form of the kernel gets on top: the step's new token of every session (one row each),
// which it appends itself, and one counter per (session, KV head), zero on entry and zero again on exit.
struct StepArgs {
    const __bf16* k_new;        // [B][Hkv][D]
    const __bf16* v_new;
    int32_t* counters;          // [B * Hkv]
};

// kStep = false: the split half of ag_attn_decode (partials to the workspace, merged by decode_merge_kernel).
// kStep = true: the whole decode step in one launch (ag_decode_step).  The workgroup whose share holds the last
// step of a (session, KV head) pair first writes the step's token into the pair's last page - the wave that will
// read that page does it, and waits for its own stores before it loads the page - and the workgroup that is
// last to finish a pair's segments (an atomic count per pair) merges them, in segment order whoever comes last,
// so the result does not depend on timing; a pair that lies inside one share is normalised and written directly.
template <bool kStep>
__global__ __launch_bounds__(256, 4) void decode_split_kernel(AttnArgs a, int32_t* __restrict__ hdr,
                                                              float* __restrict__ ws_o, float* __restrict__ ws_ml,
                                                              int pmax, StepArgs sa)
{
    __shared__ float s_o[4][16][D];     // per wave, per (padded) head: unnormalised O
    __shared__ float s_m[4][16];
    __shared__ float s_l[4][16];
    __shared__ int s_red[4];
    constexpr int kQRow = 2 * D + 16;
    __shared__ __attribute__((aligned(16))) unsigned char s_q[16 * kQRow];
    __shared__ int s_start[3];          // session holding the workgroup's first step, steps before it, its length
    __shared__ int s_arrived;           // kStep: how many of the pair's segments had been finished before this one

    const int B = a.batch, hkv = a.c.hkv, hq = a.hq;
    const int G = hq / hkv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg = blockIdx.x, W = gridDim.x;

    // ---- the plan: F, q and where this workgroup's share starts ----
    int total;
    {
        int loc = 0;
        for (int s = tid; s < B; s += 256) loc += steps_of(a.ctx_lens[s]);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) loc += __shfl_xor(loc, d);
        if (lane == 0) s_red[w] = loc;
        __syncthreads();
        total = s_red[0] + s_red[1] + s_red[2] + s_red[3];
        __syncthreads();
    }
    if (kStep) {                        // a session without context gets a row of zeros (no workgroup's share holds it)
        for (int se = wg; se < B; se += W)
            if (a.ctx_lens[se] <= 0)
                for (int idx = tid; idx < hq * D; idx += 256) ((__bf16*)a.out)[(int64_t)se * hq * D + idx] = (__bf16)0.0f;
    }
    const int F = hkv * total;
    if (F == 0) return;
    const int q = max(kMinSteps, (F + W - 1) / W);
    const int f0 = wg * q;              // q <= kMaxSteps by the launcher's choice of W: no overflow
    if (!kStep && wg == 0 && tid == 0) hdr[0] = q;
    if (f0 >= F) return;                // uniform over the workgroup
    const int f1 = min(f0 + q, F);
    {
        int carry = 0;                  // steps of the sessions before this chunk of 256
        for (int s0 = 0; s0 < B; s0 += 256) {
            const int s = s0 + tid;
            const int len = s < B ? a.ctx_lens[s] : 0;
            const int n = steps_of(len);
            int incl = n;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int t = __shfl_up(incl, d);
                if (lane >= d) incl += t;
            }
            if (lane == 63) s_red[w] = incl;
            __syncthreads();
            int woff = 0;
            for (int ww = 0; ww < w; ++ww) woff += s_red[ww];
            const int chunk = s_red[0] + s_red[1] + s_red[2] + s_red[3];
            const int excl = carry + woff + incl - n;
            if (n > 0 && hkv * excl <= f0 && f0 < hkv * (excl + n)) { s_start[0] = s; s_start[1] = excl; s_start[2] = len; }
            if (!kStep && wg == 0 && s < B) hdr[1 + s] = excl;       // workgroup 0 publishes the plan for the merge kernel
            __syncthreads();
            carry += chunk;
            if ((kStep || wg != 0) && hkv * carry > f0) break;     // found (uniform); workgroup 0 goes on publishing
        }
    }
    int s = s_start[0];
    int base = hkv * s_start[1];        // flat step at which session s starts
    int ctx = s_start[2];
    int n = steps_of(ctx);
    int g = (f0 - base) / n;
    int u = (f0 - base) - g * n;        // first step inside (s, g)

    const __bf16* kpool = (const __bf16*)a.c.k;
    const __bf16* vpool = (const __bf16*)a.c.v;
    const float sl2 = a.scale * kLog2e;

    for (int f = f0; f < f1 && s < B;) {                 // one segment per pass; every value here is uniform
        const int k = min(n - u, f1 - f);                // steps of this segment, 1 .. q
        if (k <= 0) break;                               // (only if the lengths changed under the kernel: never spin)
        const int per = (k + 3) >> 2;                    // steps per wave, at most kMaxSteps / 4 = 32
        const int my_u = u + w * per;
        const int my_n = max(0, min(per, k - w * per));

        // Everything a lane derives from its number is derived again in each segment, behind a barrier the
        // compiler cannot see through: hoisted out of this loop those values would stay in registers across
        // the step loop, which needs all 128 for the 16 loads of a step to be in flight together.
        int lane_s = lane;
        asm volatile("" : "+v"(lane_s));
        const int r = lane_s & 15, c = lane_s >> 4;
        // Row r of the first score product is slot (r & 7) of page (r >> 3) of the step; the second product takes
        // slots 8..15.  K page layout [chunk][slot][8]: lanes r = 0..7 of one lane group read 128 contiguous bytes.
        // Lane group c then owns slots (c&1)*4 + {0..3} and 8 + (c&1)*4 + {0..3} of page (c >> 1): exactly the 8
        // keys of chunk (c&1) of that value page (see v_offset), so its 16-byte V load is its P operand's partner.
        const int k_pg = r >> 3;
        const int k_off = (c * PS + (r & 7)) * 8;            // + kk * 4 * PS * 8 per k-step; + 8 * 8 for slots 8..15
        const int v_pg = c >> 1;
        const int v_off = ((c & 1) * D + r) * 8;             // value page [half][channel][8 keys]; + mb * 16 * 8 per block

        // Q of the pair's G heads goes through LDS (rows of 256 B + 16 B of padding, zero beyond G): as the B
        // operand, column = head r, k = channels kk*32 + c*8 .. +7, read when a step needs it rather than
        // held in 16 registers across the loads.
        // kStep: the segment that ends the pair also appends the step's token (position ctx - 1).  The wave whose
        // quarter holds the pair's last step writes it - 16 lanes a 16-byte piece of the key each, every lane two
        // channels of the value - and waits for these stores before it loads that step (below).
        // Every load of this prologue (Q, page ids, the new token) is issued before the first of them is used.
        const bool appends = kStep && u + k == n && w == (k - 1) / per;        // uniform over the wave
        int tid_q = tid;                                     // 256 threads: 16 heads x 16 pieces of 16 bytes
        asm volatile("" : "+v"(tid_q));
        const int head_q = tid_q >> 4, ch_q = tid_q & 15;
        u32x4 qx = {0, 0, 0, 0};
        if (head_q < G)
            qx = *reinterpret_cast<const u32x4*>((const __bf16*)a.q + ((int64_t)s * hq + (int64_t)g * G + head_q) * D + ch_q * 8);
        // physical pages of this wave's steps (lane i: page i of its run, clamped to the session's last page)
        const int last_lp = ((ctx + PS - 1) >> 4) - 1;
        int my_pid = 0;
        if (my_n > 0) my_pid = a.bt[(int64_t)s * a.max_pages + min(2 * my_u + lane_s, last_lp)];
        u32x4 new_k = {0, 0, 0, 0};
        __bf16 new_v0 = (__bf16)0.0f, new_v1 = (__bf16)0.0f;
        if (appends) {
            const __bf16* ks = sa.k_new + ((int64_t)s * hkv + g) * D;
            const __bf16* vs = sa.v_new + ((int64_t)s * hkv + g) * D;
            if (lane_s < 16) new_k = *reinterpret_cast<const u32x4*>(ks + lane_s * 8);
            new_v0 = vs[lane_s];
            new_v1 = vs[lane_s + 64];
        }
        *reinterpret_cast<u32x4*>(s_q + head_q * kQRow + ch_q * 16) = qx;
        if (appends) {
            const int slot = (ctx - 1) & (PS - 1);
            const int64_t page = __builtin_amdgcn_readlane(my_pid, last_lp - 2 * my_u);   // the run holds the last page
            __bf16* kdst = (__bf16*)a.c.k + (page * hkv + g) * (int64_t)(D * PS);
            __bf16* vdst = (__bf16*)a.c.v + (page * hkv + g) * (int64_t)(D * PS);
            if (lane_s < 16) *reinterpret_cast<u32x4*>(kdst + (lane_s * PS + slot) * 8) = new_k;
            vdst[v_offset(slot, lane_s, PS, D)] = new_v0;
            vdst[v_offset(slot, lane_s + 64, PS, D)] = new_v1;
        }

        float m = -INFINITY, lsum = 0.0f;
        f32x4 o[8];
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
        __syncthreads();                                 // Q is in LDS
        const unsigned char* q_lane = s_q + r * kQRow + c * 16;

#pragma unroll 1
        for (int st = 0; st < my_n; ++st) {
            StepRegs x;
            if (appends && st == my_n - 1) {             // the token this wave appended lies in the page loaded next
                __builtin_amdgcn_s_waitcnt(0x0070 | (0xF << 8));          // vmcnt(0): its stores have been performed
                asm volatile("" ::: "memory");
            }
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
                // all 16 loads are in flight before anything waits: left to itself the scheduler starts the
                // score product on the first keys and issues the value loads a memory latency later
                __builtin_amdgcn_sched_barrier(0);
            }
            const int tok0 = (my_u + st) * 32;
            f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const bf16x8 qk = *reinterpret_cast<const bf16x8*>(q_lane + kk * 64);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k1[kk], qk, s1, 0, 0, 0);
                s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k2[kk], qk, s2, 0, 0, 0);
            }
            // s1[i]: token tokb + i, s2[i]: token tokb + 8 + i, of head r
            const int tokb = tok0 + (c >> 1) * PS + (c & 1) * 4;
            const int keep = ctx - tokb;     // token tokb + j exists iff j < keep
            float xs[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xs[i] = (i < keep) ? s1[i] * sl2 : -INFINITY;
                xs[4 + i] = (8 + i < keep) ? s2[i] * sl2 : -INFINITY;
            }
            float mx = fmaxf(fmaxf(fmaxf(xs[0], xs[1]), fmaxf(xs[2], xs[3])), fmaxf(fmaxf(xs[4], xs[5]), fmaxf(xs[6], xs[7])));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m, mx);          // finite: token tok0 exists
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            float psum = 0.f;
            bf16x8 pb;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float p = __builtin_amdgcn_exp2f(xs[e] - m_new);
                psum += p;
                pb[e] = (__bf16)p;
            }
            lsum = lsum * alpha + psum;
            m = m_new;
            if (tok0 + 32 > ctx) {           // last, partial step: unwritten slots may hold anything, NaN included
#pragma unroll
                for (int mb = 0; mb < 8; ++mb) x.v[mb] = keep_quads(x.v[mb], keep, keep - 8);
            }
#pragma unroll
            for (int mb = 0; mb < 8; ++mb) {
                o[mb] *= alpha;
                o[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.v[mb], pb, o[mb], 0, 0, 0);
            }
        }
        lsum += __shfl_xor(lsum, 16);
        lsum += __shfl_xor(lsum, 32);

        // o[mb][i] is O^T[d = mb*16 + c*4 + i][head r]
        int lane_e = lane, tid_e = tid;                  // (as above: addresses of the merge are computed here)
        asm volatile("" : "+v"(lane_e), "+v"(tid_e));
        const int re = lane_e & 15, ce = lane_e >> 4;
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) *reinterpret_cast<f32x4*>(&s_o[w][re][mb * 16 + ce * 4]) = o[mb];
        if (ce == 0) { s_m[w][re] = m; s_l[w][re] = lsum; }
        __syncthreads();

        // the pair starts at flat step base + g n; its segments are numbered from the workgroup holding that step
        const int first_wg = (base + g * n) / q;
        const int piece = wg - first_wg;
        const int pieces = (base + g * n + n - 1) / q - first_wg + 1;
        const bool direct = kStep && pieces == 1;        // the pair lies inside this share: no partial, no merge
        if (piece < pmax) {
            for (int idx = tid_e; idx < G * D; idx += 256) {
                const int head = idx >> 7, d = idx & (D - 1);
                float ms = s_m[0][head];               // wave 0 always has a step: finite
#pragma unroll
                for (int ww = 1; ww < 4; ++ww) ms = fmaxf(ms, s_m[ww][head]);
                float acc = 0.f, l = 0.f;
#pragma unroll
                for (int ww = 0; ww < 4; ++ww) {
                    const float fw = exp2f(s_m[ww][head] - ms);   // a wave without steps has m = -inf -> 0
                    acc += fw * s_o[ww][head][d];
                    l += fw * s_l[ww][head];
                }
                const int64_t row = (int64_t)s * hq + (int64_t)g * G + head;
                if (direct) {
                    ((__bf16*)a.out)[row * D + d] = (__bf16)(acc / l);
                } else {
                    const int64_t slot = row * pmax + piece;
                    if (kStep) {                       // read by another workgroup of this launch: device-scope stores
                        store_coherent(ws_o + slot * D + d, acc);
                        if (d == 0) { store_coherent(ws_ml + slot * 2, ms); store_coherent(ws_ml + slot * 2 + 1, l); }
                    } else {
                        ws_o[slot * D + d] = acc;
                        if (d == 0) { ws_ml[slot * 2] = ms; ws_ml[slot * 2 + 1] = l; }
                    }
                }
            }
        }
        if (kStep && !direct) {
            // Count this segment in; whoever completes the pair merges all its segments, in their order.  The
            // partials were stored at device scope (they go past this XCD's caches), the barrier below waits
            // until every thread's stores have been performed before the count is raised, and the merging
            // workgroup reads them at device scope after it has seen the full count: no cache-wide write-back
            // or invalidate is needed (a device-wide fence costs a multiple of the whole step here).
            __syncthreads();
            if (tid_e == 0) s_arrived = __hip_atomic_fetch_add(&sa.counters[s * hkv + g], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (s_arrived == pieces - 1) {
                for (int idx = tid_e; idx < G * D; idx += 256) {
                    const int head = idx >> 7, d = idx & (D - 1);
                    const int64_t row = (int64_t)s * hq + (int64_t)g * G + head;
                    ((__bf16*)a.out)[row * D + d] = (__bf16)merge_partials<true>(ws_o, ws_ml, row * pmax, min(pieces, pmax), d);
                }
                if (tid_e == 0) sa.counters[s * hkv + g] = 0;      // as the next call expects it
            }
        }
        __syncthreads();                                 // s_o is rewritten by the next segment

        f += k;
        u += k;
        if (u == n) {                                    // on to the next pair
            u = 0;
            if (++g == hkv) {
                g = 0;
                base += hkv * n;
                do {
                    ++s;
                    ctx = s < B ? a.ctx_lens[s] : 0;
                    n = steps_of(ctx);
                } while (s < B && n == 0);
            }
        }
    }
}

__global__ __launch_bounds__(128) void decode_merge_kernel(AttnArgs a, const int32_t* __restrict__ hdr,
                                                           const float* __restrict__ ws_o,
                                                           const float* __restrict__ ws_ml, int pmax)
{
    const int row = blockIdx.x;                 // s * hq + h
    const int s = row / a.hq, h = row - s * a.hq;
    const int d = threadIdx.x;
    const int ctx = a.ctx_lens[s];
    __bf16* out = (__bf16*)a.out + (int64_t)row * D;
    if (ctx <= 0) { out[d] = (__bf16)0.0f; return; }
    const int q = max(1, hdr[0]), n = steps_of(ctx);
    const int first = a.c.hkv * hdr[1 + s] + (h / (a.hq / a.c.hkv)) * n;       // the pair's first flat step
    const int pieces = min(pmax, (first + n - 1) / q - first / q + 1);          // as the split kernel cuts them
    out[d] = (__bf16)merge_partials(ws_o, ws_ml, (int64_t)row * pmax, pieces, d);
}

}  // namespace

// CUs of the current device.
int device_cus()
{
    static std::atomic<int> cached[16];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return 256; }
    const bool in_table = dev >= 0 && dev < 16;
    if (in_table) { const int v = cached[dev].load(); if (v > 0) return v; }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        cus = 256;
    }
    if (in_table) cached[dev].store(cus);
    return cus;
}

// CUs the stream's launches may use: the bits of its CU mask (paper Sec. III-C: decode runs on a partition),
// the whole device if the stream has none.
int stream_cus(hipStream_t st)
{
    const int all = device_cus();
    uint32_t words[32] = {0};
    const uint32_t n_words = (uint32_t)std::min(32, (all + 31) / 32);
    if (hipExtStreamGetCUMask(st, n_words, words) != hipSuccess) { (void)hipGetLastError(); return all; }
    int n = 0;
    for (uint32_t i = 0; i < n_words; ++i) n += __builtin_popcount(words[i]);
    return n > 0 && n <= all ? n : all;
}

namespace {

// Workgroups of a launch: the shares are equal, so what matters is that every CU gets the same number of
// them, and as few as the longest share (kMaxSteps) allows: each workgroup pays the plan and each segment a
// dependent page-id read (two per CU measured 1.5 % faster than four on the whole device, and 2-4 % on
// partitions whose CU count divides the grid; a grid that leaves some CUs one workgroup short loses 4-5 %).
int workgroups_for(int64_t f_max, hipStream_t st)
{
    const int64_t unit = 2 * (int64_t)stream_cus(st);
    const int64_t need = std::max<int64_t>(1, (f_max + kMaxSteps - 1) / kMaxSteps);
    return (int)(unit * ((need + unit - 1) / unit));
}

}  // namespace

size_t decode_workspace_bytes(int batch, int hq, int d, int max_ctx)
{
    if (batch <= 0) return 0;
    return header_ints(batch) * sizeof(int32_t) + (size_t)batch * hq * pieces_max(max_ctx) * (size_t)(d + 2) * sizeof(float);
}

bool decode_mfma_supported(const AttnArgs& a)
{
    return a.c.dtype == AG_BF16 && a.c.d == D && a.c.ps == PS && (a.hq / a.c.hkv) <= 16 &&
           (((uintptr_t)a.q | (uintptr_t)a.c.k | (uintptr_t)a.c.v) % 16 == 0);
}

ag_status decode_static_scratch(void** ptr_out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = -1;
    ag_status e = hip_check(hipGetDevice(&dev), "hipGetDevice");
    if (e) return e;
    if (dev < 0 || dev >= kMaxDevices) { set_error("device %d is beyond the %d devices the static scratch is kept for", dev, kMaxDevices); return AG_ERR_UNSUPPORTED; }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {                   // each device holds its own copy of the array at its own address
        void* p = nullptr;
        if ((e = hip_check(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)"))) return e;
        if (!p) { set_error("hipGetSymbolAddress(scratch) returned a null address"); return AG_ERR_HIP; }
        ptrs[dev] = p;
    }
    *ptr_out = ptrs[dev];
    return AG_OK;
}

ag_status launch_decode_mfma(const AttnArgs& a, void* ws, hipStream_t st)
{
    const int pmax = pieces_max(a.max_ctx);
    int32_t* hdr = (int32_t*)ws;
    float* ws_o = (float*)(hdr + header_ints(a.batch));
    float* ws_ml = ws_o + (size_t)a.batch * a.hq * pmax * D;
    // Upper bound of the step count from the host-known bounds; the grid is sized so that a share is at most
    // kMaxSteps steps even if every session is max_ctx long.
    const int64_t f_max = (int64_t)a.c.hkv * a.batch * ((a.max_ctx + 31) / 32);
    if (f_max > (1 << 30)) { set_error("decode batch of %lld steps of 32 tokens is beyond one launch", (long long)f_max); return AG_ERR_INVALID_ARG; }
    if (a.max_ctx > 0) {
        const int grid = workgroups_for(f_max, st);
        // the event bracket covers both kernels of the call: the merge kernel writes the output the byte count includes
        prof_before(st);
        hipLaunchKernelGGL(decode_split_kernel<false>, dim3(grid), dim3(256), 0, st, a, hdr, ws_o, ws_ml, pmax, StepArgs{});
        ag_status e = hip_check(hipGetLastError(), "decode split launch");
        if (e) return e;
    }
    hipLaunchKernelGGL(decode_merge_kernel, dim3(a.batch * a.hq), dim3(128), 0, st, a, hdr, ws_o, ws_ml, pmax);
    prof_after(st);
    return hip_check(hipGetLastError(), "decode merge launch");
}

// ---- the whole step in one launch ----
// Workspace: a counter region of fixed size at the start - wherever the partials of a call of another shape
// may have landed, they never land here, so the counters stay zero from call to call - then the split
// kernel's workspace.
static size_t step_counter_bytes(int, int) { return AG_DECODE_STEP_COUNTER_BYTES; }

size_t decode_step_workspace_bytes(int batch, int hq, int d, int max_ctx)
{
    if (batch <= 0) return 0;
    return step_counter_bytes(batch, hq) + decode_workspace_bytes(batch, hq, d, max_ctx);
}

ag_status launch_decode_step(const AttnArgs& a, const void* k_new, const void* v_new, void* ws, hipStream_t st)
{
    if ((int64_t)a.batch * a.c.hkv * (int64_t)sizeof(int32_t) > (int64_t)AG_DECODE_STEP_COUNTER_BYTES) {
        set_error("batch * num_kv_heads = %lld exceeds the %d counters of a decode-step workspace", (long long)a.batch * a.c.hkv,
                  (int)(AG_DECODE_STEP_COUNTER_BYTES / sizeof(int32_t)));
        return AG_ERR_INVALID_ARG;
    }
    const int pmax = pieces_max(a.max_ctx);
    int32_t* counters = (int32_t*)ws;
    int32_t* hdr = (int32_t*)((unsigned char*)ws + step_counter_bytes(a.batch, a.hq));
    float* ws_o = (float*)(hdr + header_ints(a.batch));
    float* ws_ml = ws_o + (size_t)a.batch * a.hq * pmax * D;
    const int64_t f_max = (int64_t)a.c.hkv * a.batch * ((a.max_ctx + 31) / 32);
    if (f_max > (1 << 30)) { set_error("decode batch of %lld steps of 32 tokens is beyond one launch", (long long)f_max); return AG_ERR_INVALID_ARG; }
    const int grid = workgroups_for(std::max<int64_t>(f_max, 1), st);
    prof_before(st);
    hipLaunchKernelGGL(decode_split_kernel<true>, dim3(grid), dim3(256), 0, st, a, hdr, ws_o, ws_ml, pmax,
                       StepArgs{(const __bf16*)k_new, (const __bf16*)v_new, counters});
    prof_after(st);
    return hip_check(hipGetLastError(), "decode step launch");
}

}  // namespace ag
