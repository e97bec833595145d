// One launch for the decode queue of the paper's scheduler: decodes and short resume prefills together
// (paper Sec. III-A: short resume prefills are merged with decodes to improve parallelism; Algorithm 1 admits
// a request to Q_D when it is a decode or no longer than B_prefill).  bf16, head_dim 128, page 16.
//
// A session brings N >= 0 new query rows at positions P .. P + N - 1 (a decode is N = 1) that attend causally
// to the session's keys: the semantics of the resume prefill.  The work is cut the way the decode step cuts
// it, because with few query rows per session the kernel is bound by reading K and V, not by arithmetic:
//
//   plan kernel     lists the items: an item is up to R groups of tq = 16 / G consecutive rows of one session
//                   (G = query heads per KV head), so that a group's tq x G (row, head) pairs fill the 16
//                   columns of the matrix instruction that the decode step leaves mostly empty; also notes
//                   each row's session.
//   split kernel    one workgroup per (item, KV head, split of the keys the item's last row may see); the
//                   decode step's loop, with a visibility limit per column instead of per session.
//   merge kernel    one workgroup per (row, head) combines the splits in split order.
//
// K and V of a session are fetched by each of its items; items of one (session, KV head, split) are dealt to
// the same XCD (their linear workgroup ids differ by a multiple of 8 when splits * KV heads is one such), so the
// repeats are served by that XCD's L2.
#include <algorithm>

#include "attn_split_common.h"

namespace ag {

namespace {

using namespace splitk;

// plan[0] = number of items, plan[2 + 2i] = session, plan[3 + 2i] = (first row of item i) / (rows per item, `tq` here);
// row_sess[row] = session of query row `row`.  Block 0 lists the items, the other blocks the rows.
__global__ __launch_bounds__(256) void merged_plan_kernel(const int32_t* __restrict__ new_lens,
                                                          const int32_t* __restrict__ cu_new, int batch,
                                                          int total_rows, int tq, int32_t* __restrict__ plan,
                                                          int32_t* __restrict__ row_sess)
{
    if (blockIdx.x > 0) {
        const int row = (blockIdx.x - 1) * 256 + threadIdx.x;
        if (row >= total_rows) return;
        int lo = 0, hi = batch;                     // largest s with cu_new[s] <= row (empty sessions skipped)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (cu_new[mid] <= row) lo = mid; else hi = mid;
        }
        row_sess[row] = lo;
        return;
    }
    __shared__ int scan[256];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < batch; base += 256) {
        const int s = base + threadIdx.x;
        const int mine = s < batch ? (new_lens[s] + tq - 1) / tq : 0;
        scan[threadIdx.x] = mine;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {   // inclusive scan
            const int v = threadIdx.x >= off ? scan[threadIdx.x - off] : 0;
            __syncthreads();
            scan[threadIdx.x] += v;
            __syncthreads();
        }
        const int first = carry + scan[threadIdx.x] - mine;
        for (int i = 0; i < mine; ++i) {
            plan[2 + 2 * (first + i)] = s;
            plan[3 + 2 * (first + i)] = i;
        }
        __syncthreads();
        if (threadIdx.x == 255) carry += scan[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) { plan[0] = carry; plan[1] = tq; }
}

// kSteps: steps of 32 keys a wave may walk; the split size is 128 * kSteps keys.
// R: column groups per item.  An item is R * tq rows; each K / V step is loaded once and used by the R groups
// one after the other, which divides the number of times a session's keys are fetched by R at the price of
// R times the accumulators (fewer waves per SIMD).
template <int kSteps, int R>
__global__ __launch_bounds__(256, R == 1 ? 4 : 2) void merged_split_kernel(AttnArgs a, float* __restrict__ ws_o,
                                                                           float* __restrict__ ws_ml,
                                                                           const int32_t* __restrict__ plan,
                                                                           int n_splits_max, int tq)
{
    constexpr int kSplit = 128 * kSteps;
    __shared__ float s_o[4][16][D];     // per wave, per column of one group: unnormalised O
    __shared__ float s_m[4][16];
    __shared__ float s_l[4][16];

    const int split = blockIdx.x, g = blockIdx.y, item = blockIdx.z;
    if (item >= plan[0]) return;
    const int rows_item = R * tq;
    const int s = plan[2 + 2 * item];
    const int t0 = plan[3 + 2 * item] * rows_item;   // first row of the item within the session's chunk
    const int N = a.new_lens[s];
    const int P = a.prefix_lens ? a.prefix_lens[s] : 0;
    const int nt = min(rows_item, N - t0);           // rows of this item, >= 1
    const int ctx_all = P + N;                       // slots below this hold tokens
    const int ctx = P + t0 + nt;                     // keys the item's last row may see
    const int part = part_tokens(ctx, kSplit);
    const int start = split * part;
    if (start >= ctx) return;                        // uniform over the workgroup
    const int wave_tok = part >> 2;

    const int hkv = a.c.hkv, hq = a.hq;
    const int G = hq / hkv;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, c = lane >> 4;
    const int wstart = start + w * wave_tok;

    const __bf16* kpool = (const __bf16*)a.c.k;
    const __bf16* vpool = (const __bf16*)a.c.v;

    // column r of group j = (row j * tq + r / G of the item, head r % G of the KV head's group); columns
    // without a row carry a zero query and the visibility of the item's last row
    const int col_row = r / G, col_head = r - col_row * G;
    int pos[R];
    bf16x8 qf[R][4];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int row = j * tq + col_row;
        const bool on = col_row < tq && row < nt;
        pos[j] = P + t0 + (on ? row : nt - 1);
        const int64_t q_row = (int64_t)a.cu_new[s] + t0 + (on ? row : 0);
        const __bf16* qrow = (const __bf16*)a.q + (q_row * hq + (int64_t)g * G + col_head) * D + c * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 x = ld16(qrow + kk * 32);
            if (!on) x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qf[j][kk] = x;
        }
    }

    const int n_pages_ctx = (ctx + PS - 1) >> 4;
    int my_pid;
    {
        const int lp = min((wstart >> 4) + (lane & (2 * kSteps - 1)), n_pages_ctx - 1);
        my_pid = a.bt[(int64_t)s * a.max_pages + lp];
    }
    const int n_steps = wstart < ctx ? min(wave_tok >> 5, (ctx - wstart + 31) >> 5) : 0;   // uniform over the wave

    const float sl2 = a.scale * kLog2e;
    float m[R], lsum[R];
    f32x4 o[R][8];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        m[j] = -INFINITY;
        lsum[j] = 0.0f;
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) o[j][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // operand addressing as in the decode step: score row r is slot (r & 7) of page (r >> 3) of the step, the
    // second score product takes slots 8..15; lane group c owns the 8 keys of value chunk (c & 1) of page (c >> 1)
    const int k_pg = r >> 3;
    const int k_off = (c * PS + (r & 7)) * 8;
    const int v_pg = c >> 1;
    const int v_off = ((c & 1) * D + r) * 8;

#pragma unroll
    for (int st = 0; st < kSteps; ++st) {
        if (st < n_steps) {
            StepRegs x;
            {
                const int64_t pA = __builtin_amdgcn_readlane(my_pid, 2 * st);
                const int64_t pB = __builtin_amdgcn_readlane(my_pid, 2 * st + 1);
                const __bf16* kp = kpool + ((k_pg ? pB : pA) * hkv + g) * (int64_t)(D * PS) + k_off;
                const __bf16* vp = vpool + ((v_pg ? pB : pA) * hkv + g) * (int64_t)(D * PS) + v_off;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    x.k1[kk] = ld16(kp + kk * 4 * PS * 8);
                    x.k2[kk] = ld16(kp + kk * 4 * PS * 8 + 64);
                }
#pragma unroll
                for (int mb = 0; mb < 8; ++mb) x.v[mb] = ld16(vp + mb * 16 * 8);
            }
            const int tok0 = wstart + st * 32;
            const int tokb = tok0 + (c >> 1) * PS + (c & 1) * 4;
#pragma unroll
            for (int j = 0; j < R; ++j) {
                f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k1[kk], qf[j][kk], s1, 0, 0, 0);
                    s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.k2[kk], qf[j][kk], s2, 0, 0, 0);
                }
                // s1[i]: key tokb + i, s2[i]: key tokb + 8 + i, of column r
                const int keep = pos[j] + 1 - tokb;  // key tokb + i is visible to this column iff i < keep
                float xs[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    xs[i] = (i < keep) ? s1[i] * sl2 : -INFINITY;
                    xs[4 + i] = (8 + i < keep) ? s2[i] * sl2 : -INFINITY;
                }
                float mx = fmaxf(fmaxf(fmaxf(xs[0], xs[1]), fmaxf(xs[2], xs[3])), fmaxf(fmaxf(xs[4], xs[5]), fmaxf(xs[6], xs[7])));
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m[j], mx);
                // a column may see none of this wave's keys so far (its row lies before them): keep the exponents finite
                const float m_ref = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f(m[j] - m_ref);
                float psum = 0.f;
                bf16x8 pb;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float p = __builtin_amdgcn_exp2f(xs[e] - m_ref);
                    psum += p;
                    pb[e] = (__bf16)p;
                }
                lsum[j] = lsum[j] * alpha + psum;
                m[j] = m_new;
                if (j == 0 && tok0 + 32 > ctx_all) {   // slots past the session's last token may hold anything, NaN included
                    const int keep_v = ctx_all - tokb;
#pragma unroll
                    for (int mb = 0; mb < 8; ++mb) x.v[mb] = keep_quads(x.v[mb], keep_v, keep_v - 8);
                }
#pragma unroll
                for (int mb = 0; mb < 8; ++mb) {
                    o[j][mb] *= alpha;
                    o[j][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x.v[mb], pb, o[j][mb], 0, 0, 0);
                }
            }
        }
    }

    // the four waves' partials of one group at a time through LDS
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int rows_here = min(tq, nt - j * tq);          // rows of group j; uniform over the workgroup
        if (rows_here <= 0) break;
        float l = lsum[j];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (j > 0) __syncthreads();                          // the previous group's readers are done
        // o[j][mb][i] is O^T[d = mb*16 + c*4 + i][column r]
#pragma unroll
        for (int mb = 0; mb < 8; ++mb) *reinterpret_cast<f32x4*>(&s_o[w][r][mb * 16 + c * 4]) = o[j][mb];
        if (c == 0) { s_m[w][r] = m[j]; s_l[w][r] = l; }
        __syncthreads();
        const int n_cols = rows_here * G;
        for (int idx = threadIdx.x; idx < n_cols * D; idx += 256) {
            const int col = idx >> 7, d = idx & (D - 1);
            float ms = s_m[0][col];
#pragma unroll
            for (int ww = 1; ww < 4; ++ww) ms = fmaxf(ms, s_m[ww][col]);
            float acc = 0.f, lt = 0.f;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                const float mw = s_m[ww][col];
                const float f = mw == -INFINITY ? 0.f : exp2f(mw - ms);    // a wave that saw no key of this column
                acc += f * s_o[ww][col][d];
                lt += f * s_l[ww][col];
            }
            const int crow = col / G, chead = col - crow * G;
            const int64_t slot = (((int64_t)a.cu_new[s] + t0 + j * tq + crow) * hq + (int64_t)g * G + chead) * n_splits_max + split;
            ws_o[slot * D + d] = acc;
            if (d == 0) { ws_ml[slot * 2] = ms; ws_ml[slot * 2 + 1] = lt; }
        }
    }
}

__global__ __launch_bounds__(128) void merged_merge_kernel(AttnArgs a, const float* __restrict__ ws_o,
                                                           const float* __restrict__ ws_ml,
                                                           const int32_t* __restrict__ row_sess, int n_splits_max,
                                                           int split_tokens, int rows_item)
{
    const int64_t rh = blockIdx.x;                 // row * hq + head
    const int row = (int)(rh / a.hq);
    const int d = threadIdx.x;
    const int s = row_sess[row];
    const int t = row - a.cu_new[s];
    const int N = a.new_lens[s];
    const int P = a.prefix_lens ? a.prefix_lens[s] : 0;
    const int t0 = (t / rows_item) * rows_item;
    const int ctx = P + t0 + min(rows_item, N - t0);      // as the split kernel cut the row's item
    const int part = part_tokens(ctx, split_tokens);
    const int n = (ctx + part - 1) / part;
    const int64_t base = rh * n_splits_max;
    float ms = -INFINITY;
    for (int i = 0; i < n; ++i) ms = fmaxf(ms, ws_ml[(base + i) * 2]);     // finite: key 0 is visible to every row
    float acc = 0.f, l = 0.f;
    for (int i = 0; i < n; ++i) {                  // fixed order: reproducible
        const float f = exp2f(ws_ml[(base + i) * 2] - ms);
        acc += f * ws_o[(base + i) * D + d];
        l += f * ws_ml[(base + i) * 2 + 1];
    }
    ((__bf16*)a.out)[rh * D + d] = (__bf16)(acc / l);
}

inline int rows_per_item(int hq, int hkv) { return 16 / (hq / hkv); }

inline int choose_split(int items, int hkv, int max_ctx)
{
    const int64_t want = 4 * 256;            // workgroups, counting contexts at about 60 % of max_ctx
    for (int split = 2048; split > kMinSplit; split >>= 1) {
        const int64_t wgs = (int64_t)items * hkv * ((6 * (int64_t)max_ctx / 10 + split - 1) / split);
        if (wgs >= want) return split;
    }
    return kMinSplit;
}

struct Layout { size_t o_floats, ml_floats, plan_ints, row_ints; };
inline Layout layout(int total_rows, int hq, int max_ctx)
{
    const size_t nsm = (size_t)splits_for(max_ctx, kMinSplit);
    return {(size_t)total_rows * hq * nsm * D, (size_t)total_rows * hq * nsm * 2, 2 + 2 * (size_t)total_rows, (size_t)total_rows};
}

}  // namespace

size_t merged_workspace_bytes(int total_rows, int hq, int max_ctx)
{
    const Layout L = layout(total_rows, hq, max_ctx);
    return (L.o_floats + L.ml_floats + L.plan_ints + L.row_ints) * 4;
}

bool merged_mfma_supported(const AttnArgs& a)
{
    const int G = a.hq / a.c.hkv;
    return a.c.dtype == AG_BF16 && a.c.d == D && a.c.ps == PS && G <= 16 &&
           (((uintptr_t)a.q | (uintptr_t)a.c.k | (uintptr_t)a.c.v) % 16 == 0);
}

template <int R>
static void launch_split(int split, dim3 grid, hipStream_t st, const AttnArgs& a, float* ws_o, float* ws_ml,
                         const int32_t* plan, int nsm, int tq)
{
    switch (split) {
        case 2048: hipLaunchKernelGGL((merged_split_kernel<16, R>), grid, dim3(256), 0, st, a, ws_o, ws_ml, plan, nsm, tq); break;
        case 1024: hipLaunchKernelGGL((merged_split_kernel<8, R>), grid, dim3(256), 0, st, a, ws_o, ws_ml, plan, nsm, tq); break;
        case 512:  hipLaunchKernelGGL((merged_split_kernel<4, R>), grid, dim3(256), 0, st, a, ws_o, ws_ml, plan, nsm, tq); break;
        default:   hipLaunchKernelGGL((merged_split_kernel<2, R>), grid, dim3(256), 0, st, a, ws_o, ws_ml, plan, nsm, tq); break;
    }
}

ag_status launch_merged_mfma(const AttnArgs& a, void* ws, hipStream_t st)
{
    if (a.total_rows <= 0) return AG_OK;
    const int tq = rows_per_item(a.hq, a.c.hkv);
    // Two column groups per item as soon as some session may bring more rows than one group holds: its keys
    // are then fetched half as often.  A batch of decodes only keeps one group (and twice the waves per SIMD).
#ifdef AG_MERGED_FORCE_R
    const int R = AG_MERGED_FORCE_R;
#else
    const int R = a.max_new > tq ? 2 : 1;
#endif
    const int rows_item = R * tq;
    // every item has at least one row, and a session of N rows has ceil(N / rows_item) items
    const int64_t items_max = std::min<int64_t>(a.total_rows, ((int64_t)a.total_rows + (int64_t)a.batch * (rows_item - 1)) / rows_item);
    if (items_max > 65535 || a.c.hkv > 65535) { set_error("too many items (%lld) or KV heads for one launch grid", (long long)items_max); return AG_ERR_INVALID_ARG; }
    const int split = choose_split((int)items_max, a.c.hkv, a.max_ctx);
    const int nsm = splits_for(a.max_ctx, split);
    const Layout L = layout(a.total_rows, a.hq, a.max_ctx);
    float* ws_o = (float*)ws;
    float* ws_ml = ws_o + L.o_floats;
    int32_t* plan = (int32_t*)(ws_ml + L.ml_floats);
    int32_t* row_sess = plan + L.plan_ints;

    hipLaunchKernelGGL(merged_plan_kernel, dim3(1 + (a.total_rows + 255) / 256), dim3(256), 0, st, a.new_lens, a.cu_new,
                       a.batch, a.total_rows, rows_item, plan, row_sess);
    ag_status e = hip_check(hipGetLastError(), "merged plan launch");
    if (e) return e;
    const dim3 grid(nsm, a.c.hkv, (unsigned)items_max);
    prof_before(st);
    if (R == 2) launch_split<2>(split, grid, st, a, ws_o, ws_ml, plan, nsm, tq);
    else launch_split<1>(split, grid, st, a, ws_o, ws_ml, plan, nsm, tq);
    prof_after(st);
    if ((e = hip_check(hipGetLastError(), "merged split launch"))) return e;
    hipLaunchKernelGGL(merged_merge_kernel, dim3((unsigned)((int64_t)a.total_rows * a.hq)), dim3(128), 0, st, a, ws_o, ws_ml,
                       row_sess, nsm, split, rows_item);
    return hip_check(hipGetLastError(), "merged merge launch");
}

}  // namespace ag
