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
//   split kernel, one workgroup (4 waves) per (session, KV head, split).  A session's context is cut into
//   n = ceil(ctx / split size) equal parts (rounded up to 128 tokens), so no workgroup is left with a sliver;
//   each wave owns a quarter of a part and walks it 32 tokens (two pages) at a time:
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
//   (m, l, O) per query head to the workspace;
//
//   merge kernel, one workgroup per (session, query head): combines the
//   partials of all splits in split order (reproducible) and writes bf16.
#include "attn_split_common.h"

namespace ag {

namespace {

using namespace splitk;

// kSteps: steps of 32 tokens a wave may walk; the split size is 128 * kSteps tokens.
template <int kSteps>
__global__ __launch_bounds__(256, 2) void decode_split_kernel(AttnArgs a, float* __restrict__ ws_o,
                                                              float* __restrict__ ws_ml, int n_splits_max)
{
    static_assert(kSteps >= 1 && kSteps <= 16, "a wave walks 1..16 steps of 32 tokens");
    constexpr int kSplit = 128 * kSteps;
    __shared__ float s_o[4][16][D];     // per wave, per (padded) head: unnormalised O
    __shared__ float s_m[4][16];
    __shared__ float s_l[4][16];

    // Workgroups are dealt to the 8 XCDs round-robin in linear order (x fastest).  Short sessions only have
    // the low split numbers, so if blockIdx.x were the split itself the XCDs that draw the low numbers would
    // get all the work of short sessions on top of their share of long ones (with 8 splits: everything on
    // one XCD per split).  Rotating the split by head and session spreads them evenly.
    const int g = blockIdx.y, s = blockIdx.z;
    const int split = (int)((blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x);
    const int ctx = a.ctx_lens[s];
    if (ctx <= 0) return;
    const int part = part_tokens(ctx, kSplit);
    const int start = split * part;
    if (start >= ctx) return;            // uniform over the workgroup
    const int wave_tok = part >> 2;      // a multiple of 32, at most 32 * kSteps

    const int hkv = a.c.hkv, hq = a.hq;
    const int G = hq / hkv;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, c = lane >> 4;
    const int wstart = start + w * wave_tok;

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

    // physical pages of this wave's logical pages (clamped to the session's last page)
    const int n_pages_ctx = (ctx + PS - 1) >> 4;
    int my_pid;
    {
        const int lp = min((wstart >> 4) + (lane & (2 * kSteps - 1)), n_pages_ctx - 1);
        my_pid = a.bt[(int64_t)s * a.max_pages + lp];
    }
    const int n_steps = wstart < ctx ? min(wave_tok >> 5, (ctx - wstart + 31) >> 5) : 0;   // uniform over the wave

    const float sl2 = a.scale * kLog2e;
    float m = -INFINITY, lsum = 0.0f;
    f32x4 o[8];
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Row r of the first score product is slot (r & 7) of page (r >> 3) of the step; the second product takes
    // slots 8..15.  K page layout [chunk][slot][8]: lanes r = 0..7 of one lane group read 128 contiguous bytes.
    // Lane group c then owns slots (c&1)*4 + {0..3} and 8 + (c&1)*4 + {0..3} of page (c >> 1): exactly the 8
    // keys of chunk (c&1) of that value page (see v_offset), so its 16-byte V load is its P operand's partner.
    const int k_pg = r >> 3;
    const int k_off = (c * PS + (r & 7)) * 8;            // + kk * 4 * PS * 8 per k-step; + 8 * 8 for slots 8..15
    const int v_pg = c >> 1;
    const int v_off = ((c & 1) * D + r) * 8;             // value page [half][channel][8 keys]; + mb * 16 * 8 per block

    auto load_step = [&](int st, StepRegs& x) {
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
    };

    auto compute_step = [&](int st, StepRegs& x) {
        const int tok0 = wstart + st * 32;
        f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k1[kk], qf[kk], s1, 0, 0, 0);
            s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k2[kk], qf[kk], s2, 0, 0, 0);
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
    };

#if AG_DECODE_PREFETCH
    StepRegs buf[2];
    if (n_steps > 0) load_step(0, buf[0]);
#pragma unroll
    for (int st = 0; st < kSteps; ++st) {
        if (st < n_steps) {
            if (st + 1 < kSteps && st + 1 < n_steps) load_step(st + 1, buf[(st + 1) & 1]);
            compute_step(st, buf[st & 1]);
        }
    }
#else
#pragma unroll
    for (int st = 0; st < kSteps; ++st) {
        if (st < n_steps) {
            StepRegs x;
            load_step(st, x);
            compute_step(st, x);
        }
    }
#endif
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
                                                           const float* __restrict__ ws_ml, int n_splits_max,
                                                           int split_tokens)
{
    const int row = blockIdx.x;                 // s * hq + h
    const int s = row / a.hq;
    const int d = threadIdx.x;
    const int ctx = a.ctx_lens[s];
    __bf16* out = (__bf16*)a.out + (int64_t)row * D;
    if (ctx <= 0) { out[d] = (__bf16)0.0f; return; }
    const int part = part_tokens(ctx, split_tokens);
    const int n = (ctx + part - 1) / part;               // parts that exist, as the split kernel cuts them
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

// Split size for a launch: as long as possible (each workgroup pays a fixed start-up of three dependent reads)
// while the launch still has a few workgroups per CU to balance with.  Only host-known bounds are available.
inline int choose_split(int batch, int hkv, int max_ctx)
{
    const int64_t want = 4 * 256;            // workgroups, counting sessions at about 60 % of max_ctx
    for (int split = 2048; split > kMinSplit; split >>= 1) {
        const int64_t wgs = (int64_t)batch * hkv * ((6 * (int64_t)max_ctx / 10 + split - 1) / split);
        if (wgs >= want) return split;
    }
    return kMinSplit;
}

}  // namespace

size_t decode_workspace_bytes(int batch, int hq, int d, int max_ctx)
{
    return (size_t)batch * hq * splits_for(max_ctx, kMinSplit) * (size_t)(d + 2) * sizeof(float);
}

bool decode_mfma_supported(const AttnArgs& a)
{
    return a.c.dtype == AG_BF16 && a.c.d == D && a.c.ps == PS && (a.hq / a.c.hkv) <= 16 &&
           (((uintptr_t)a.q | (uintptr_t)a.c.k | (uintptr_t)a.c.v) % 16 == 0);
}

ag_status launch_decode_mfma(const AttnArgs& a, void* ws, hipStream_t st)
{
#ifdef AG_DECODE_FORCE_SPLIT
    const int split = AG_DECODE_FORCE_SPLIT;
#else
    const int split = choose_split(a.batch, a.c.hkv, a.max_ctx);
#endif
    const int nsm = splits_for(a.max_ctx, split);
    float* ws_o = (float*)ws;
    float* ws_ml = ws_o + (size_t)a.batch * a.hq * nsm * D;
    if (a.batch > 65535 || a.c.hkv > 65535) { set_error("batch or KV heads beyond one launch grid"); return AG_ERR_INVALID_ARG; }
    if (a.max_ctx > 0) {
        const dim3 grid(nsm, a.c.hkv, a.batch);
        prof_before(st);
        switch (split) {
            case 2048: hipLaunchKernelGGL(decode_split_kernel<16>, grid, dim3(256), 0, st, a, ws_o, ws_ml, nsm); break;
            case 1024: hipLaunchKernelGGL(decode_split_kernel<8>, grid, dim3(256), 0, st, a, ws_o, ws_ml, nsm); break;
            case 512:  hipLaunchKernelGGL(decode_split_kernel<4>, grid, dim3(256), 0, st, a, ws_o, ws_ml, nsm); break;
            default:   hipLaunchKernelGGL(decode_split_kernel<2>, grid, dim3(256), 0, st, a, ws_o, ws_ml, nsm); break;
        }
        prof_after(st);
        ag_status e = hip_check(hipGetLastError(), "decode split launch");
        if (e) return e;
    }
    hipLaunchKernelGGL(decode_merge_kernel, dim3(a.batch * a.hq), dim3(128), 0, st, a, ws_o, ws_ml, nsm, split);
    return hip_check(hipGetLastError(), "decode merge launch");
}

}  // namespace ag
