// Cold and resume prefill over a paged KV cache, bf16, head_dim 128, page 16
// (paper Sec. I and Sec. II-A: a cold prefill is full causal attention over
// the prompt; a resume prefill appends a chunk to a cached context, so row i
// of a session with P cached tokens sees keys 0 .. P + i.  Cold is P = 0.)
//
// A dense contraction, bound by the matrix cores: 4 * D flop per visible
// (query, key) pair and head.  One workgroup of NW waves (4 or 8) owns 32 * NW
// query rows of one session: consecutive tokens of one query head, or - when
// the KV-head group has 2, 4 or 8 query heads - fewer tokens of all the
// group's heads, which share K and V (see the kernel's GP parameter); each
// wave owns 32 tokens of one head and keeps their Q in registers.  Keys and
// values are taken 64 at a time (4 pages) and staged through LDS by direct
// global-to-LDS loads:
//
//   S^T[key][query] = K[key][:] . Q[query][:]      2 x 8 MFMA 32x32x16
//   softmax weights per query column (reference m, running sum l, exp2)
//   O^T[d][query]  += V^T[d][key] . P^T[key][query]  4 x 4 MFMA 32x32x16
//
// Computing the transposed score tile puts one query in one lane (plus its
// partner lane + 32), so the row max / sum need a single cross-lane step,
// and the 8 scores a lane holds for one k-step of the second product are
// already its B operand: P never leaves registers.  The pools' page layouts
// are the LDS tile layouts (K chunk-major, V transposed in 8-key chunks in the
// slot order the score tile produces), so a tile is copied as contiguous runs,
// 16-byte operand reads are conflict free and every operand address is the
// lane's base plus a constant.
//
// The per-element softmax work on the vector ALUs is about as long as the
// matrix work (one exp per 512 flop), so iteration t of a wave interleaves,
// instruction by instruction, O += V(t-1).P(t-1) (matrix) with
// P(t) = exp2(S(t) - m) (vector), after S(t) = K(t).Q^T.  m is a reference,
// not the running maximum: the common case takes the weights under the current
// m and only checks afterwards that none came out large; a wave's first tile
// and a failed check take an ordered path that finds the row maxima, rescales
// O and l when a maximum outgrew m by more than 2^8, and recomputes the weights.
// Tiles wholly above a wave's rows are skipped; the tiles on the diagonal are
// masked before the weights are taken.
//
// Workgroups are numbered so that the XCD a workgroup lands on (id % 8) owns a
// contiguous range of KV heads, and inside it session-major, longest query
// tile first: the workgroups resident together read one session's K/V for one
// KV head, which then stays in that XCD's L2.  The grid lists the batch's real
// tiles only (each workgroup finds its tile from the chunk lengths): empty
// workgroups are not free, the dispatcher takes as long over them as over
// the others.
#include <algorithm>
#include <atomic>

#include "ag_internal.h"
#include "attn_tile32.h"
#include "lds_dma.h"

namespace ag {

namespace {

using namespace tile32;

// V stages: 2 (V(t) requested while V(t-1) is used).  A third stage (V(t+1) requested an iteration earlier) is
// supported by the loop but measured no faster, so both workgroup shapes use 80 KiB: two 4-wave workgroups or
// one 8-wave workgroup per CU.
constexpr int v_stages(int) { return 2; }
// The 8-wave form also keeps two windows of 64 page ids (16 key tiles each) of the session's block-table row in
// LDS, see the kernel; the 4-wave form has no room for them (two workgroups of 80 KiB fill a CU's LDS).
constexpr int kIdWindow = 64;
constexpr bool ids_in_lds(int nw) { return nw == 8; }
constexpr int lds_bytes(int nw) { return (kKStages + v_stages(nw)) * kTile + (ids_in_lds(nw) ? 2 * kIdWindow * 4 : 0); }
constexpr int kWavesPerSimd = 2;        // 205 registers per lane

// NW waves per workgroup (4 or 8), 32 query rows each.  Eight waves halve the K/V bytes moved per flop (a tile
// is shared by twice the rows) at the price of coarser query tiles.
// GP: query heads per workgroup.  GP = 1: the NW waves are 32 * NW consecutive tokens of one head.  GP = G (the
// heads of a KV-head group, which share K and V): wave w is head w % GP of tokens 32 * (w / GP) .. + 31, so the
// workgroup covers 32 * NW / GP tokens of all G heads.  The rows per K/V tile are the same, but a chunk is cut
// every 32 * NW / GP tokens instead of every 32 * NW (ragged chunks fill their last tile better) and all waves
// of a workgroup end within one tile of each other on the diagonal.
template <int NW, int GP>
__global__ __launch_bounds__(64 * NW, kWavesPerSimd) void prefill_mfma_kernel(AttnArgs a, int tiles_max,
                                                                                         int per_xcd, int64_t total_work)
{
    static_assert(NW % GP == 0, "the heads of a group share the workgroup's waves evenly");
    constexpr int BM = 32 * NW / GP;        // tokens per workgroup
    constexpr int kPer = 16 / NW;           // direct-load instructions per wave for a K tile, and for a V tile
    constexpr int kVStages = v_stages(NW);
    constexpr int kVLead = kVStages - 2;    // V(t + kVLead) is requested in iteration t
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // ---- which (session, head, query tile) ----
    const int xcd = blockIdx.x & 7, ord = blockIdx.x >> 3;
    const int64_t wk = (int64_t)xcd * per_xcd + ord;
    if (wk >= total_work) return;
    const int hkv = a.c.hkv, hq = a.hq, G = hq / hkv;
    // Work order: KV head, then session, then query tile (longest first), then (GP = 1) the G heads of the group.
    // The grid holds `tiles_max` tiles per KV head, a host-side bound on sum_s ceil(N_s / BM); which (session,
    // tile) the workgroup's tile index means follows from the lengths, which every wave scans for itself (lane l
    // of a pass holds session 64 * pass + l).  A grid of batch x ceil(max_new / BM) tiles would be mostly empty
    // workgroups when chunk lengths differ much, and launching a workgroup of this size takes the dispatcher of
    // an XCD most of a microsecond, whether it has work or not.
    const int hpw = GP == 1 ? G : 1;                // workgroups a tile of tokens takes
    const int per_head = tiles_max * hpw;
    const int g = (int)(wk / per_head);
    const int rem = (int)(wk % per_head);
    const int j = rem / hpw;                        // tile index among the KV head's tiles
    int s = -1, qt = 0, N = 0, P = 0, row0 = 0;
    {
        const int ln = threadIdx.x & 63;
        int before = 0;                             // tiles of the sessions of earlier passes
        for (int s0 = 0; s0 < a.batch && s < 0; s0 += 256) {
            // four passes' lengths are fetched together, and with them the prefix length and the row offset of
            // every session: whichever session the tile turns out to belong to, no second round trip follows
            int lens[4], pre[4], cu[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ss = s0 + 64 * k + ln;
                const bool in = ss < a.batch;
                lens[k] = in ? a.new_lens[ss] : 0;
                pre[k] = in && a.prefix_lens ? a.prefix_lens[ss] : 0;
                cu[k] = in ? a.cu_new[ss] : 0;
            }
            // A batch that fits one pass is walked longest context first: workgroups start in list order, and a
            // launch ends sooner when the tiles left for its end are the short ones (each has P + position keys
            // to go through).  Every wave ranks the sessions itself; equal contexts keep the given order.
            int sess = ln;                          // the session this lane's entry describes
            if (a.batch <= 64) {
                const int key = ln < a.batch ? pre[0] + lens[0] : -1;
                const int key0 = __builtin_amdgcn_readlane(key, 0);
                if (__builtin_amdgcn_ballot_w64(ln < a.batch && key != key0) != 0) {       // uniform
                    int rank = 0;                   // sessions ahead of this one: longer, or as long and earlier
                    for (int o = 0; o < a.batch; ++o) {
                        const int ko = __builtin_amdgcn_readlane(key, o);
                        rank += (ko > key || (ko == key && o < ln)) ? 1 : 0;
                    }
                    if (ln >= a.batch) rank = ln;   // entries without a session stay where they are
                    sess = __builtin_amdgcn_ds_permute(rank << 2, sess);
                    lens[0] = __builtin_amdgcn_ds_permute(rank << 2, lens[0]);
                    pre[0] = __builtin_amdgcn_ds_permute(rank << 2, pre[0]);
                    cu[0] = __builtin_amdgcn_ds_permute(rank << 2, cu[0]);
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (s >= 0) break;                  // uniform
                const int len = lens[k];
                const int cnt = (len + BM - 1) / BM;
                int incl = cnt;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const int t = __shfl_up(incl, d);
                    if (ln >= d) incl += t;
                }
                const int pass_total = __builtin_amdgcn_readlane(incl, 63);
                if (j < before + pass_total) {      // uniform
                    const unsigned long long hit = __builtin_amdgcn_ballot_w64(j < before + incl);
                    const int l = __builtin_ctzll(hit);              // first session whose tiles reach past j
                    s = s0 + 64 * k + (k == 0 ? __builtin_amdgcn_readlane(sess, l) : l);
                    N = __builtin_amdgcn_readlane(len, l);
                    P = __builtin_amdgcn_readlane(pre[k], l);
                    row0 = __builtin_amdgcn_readlane(cu[k], l);
                    qt = before + __builtin_amdgcn_readlane(incl, l) - 1 - j;   // the session's tiles, longest first
                }
                before += pass_total;
            }
        }
    }
    if (s < 0) return;                              // beyond the batch's tiles
    const int q0 = qt * BM;
    const int ctx = P + N;
    const int64_t t_base = (int64_t)row0 + q0;

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int wu = __builtin_amdgcn_readfirstlane(w);           // the same value, known to be uniform: used only
                                                                 // where a scalar is required (page ids, M0)
    const int n = lane & 31, hi = lane >> 5;
    const int rows_wg = min(BM, N - q0);            // valid tokens of this workgroup
    const int qrow0 = 32 * (w / GP);                // first token of this wave inside the tile
    const int h = g * G + (GP == 1 ? rem % G : w % GP);     // this wave's query head
    const int rows_w = max(0, min(32, rows_wg - qrow0));

    const int n_tiles = (P + q0 + rows_wg - 1) / BN + 1;                        // tiles the workgroup stages
    const int wave_tiles = rows_w > 0 ? (P + q0 + qrow0 + rows_w - 1) / BN + 1 : 0;   // tiles this wave uses
    const int first_masked = (P + q0 + qrow0 + 1) / BN;   // first tile holding a key this wave's row 0 may not see

    const __bf16* kpool = (const __bf16*)a.c.k;
    const __bf16* vpool = (const __bf16*)a.c.v;
    // the block table is read-only for the kernel's lifetime: reading it through the constant address space
    // lets the (uniform) page-id loads be scalar loads, which use their own counter
    typedef const __attribute__((address_space(4))) int32_t* cptr_t;
    const cptr_t bt = (cptr_t)(uintptr_t)(a.bt + (int64_t)s * a.max_pages);
    const int last_page = (ctx - 1) >> 4;

    // ---- Q^T as B operand: column n = query row, k-step ks covers channels ks*16 + hi*8 .. +7 ----
    bf16x8 qf[8];
    {
        const int row = min(qrow0 + n, rows_wg - 1);
        const __bf16* qp = (const __bf16*)a.q + ((t_base + row) * hq + h) * D + hi * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    // ---- tile requests: direct global-to-LDS loads, 4 + 4 wave-wide instructions per wave and tile ----
    unsigned char* const k_lds = lds;                       // K tile t lives at k_lds + (t % 3) * kTile
    unsigned char* const v_lds = lds + kKStages * kTile;    // V tile t lives at v_lds + (t % kVStages) * kTile
    const int kpg = lane >> 4, kslot = lane & 15;           // K: lane = key of the tile (page, slot)
    const int kmask[4] = {kpg == 0 ? -1 : 0, kpg == 1 ? -1 : 0, kpg == 2 ? -1 : 0, kpg == 3 ? -1 : 0};

    // Physical pages of a tile.  Scalar form (the prologue, and the 4-wave kernel throughout): scalar loads (the
    // index is uniform), fetched one iteration before the tile's data is requested.  A scalar load in flight
    // costs more than its latency, though: it shares a counter with the LDS operand reads and returns out of
    // order, so while one is pending every wait for an operand becomes a wait for everything.  The 8-wave
    // kernel therefore keeps the ids in LDS: wave 0 brings the session's block-table row in windows of 64
    // pages (16 key tiles) by one direct load each, two windows resident, and every lane reads the id it needs
    // (its own page of the K tile, the wave's page of the V tile) with an ordinary LDS read.
    constexpr bool kLdsIds = ids_in_lds(NW);
    struct Pages { int k; int v; };                            // k: this LANE's page of the K tile; v: the wave's page of the V tile
    const int v_page = (wu * kPer) / 4;                        // page of a V tile this wave brings in (4 runs per page)
    auto pages_scalar = [&](int tk, int tv, Pages& pg) {
        int pid[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pid[i] = bt[min(tk * 4 + i, last_page)];
        // this lane's page among the four (uniform) ids, by masks: a chain of ?: here compiles to branches
        pg.k = (pid[0] & kmask[0]) | (pid[1] & kmask[1]) | (pid[2] & kmask[2]) | (pid[3] & kmask[3]);
        pg.v = bt[min(tv * 4 + v_page, last_page)];
    };
    const int32_t* const id_lds = reinterpret_cast<const int32_t*>(lds + (kKStages + kVStages) * kTile);
    // window w = logical pages [64 w, 64 w + 64), clamped to the session's last page, into slot w & 1
    auto refill_ids = [&](int win) {
        const int lp = min(win * kIdWindow + lane, last_page);
        load_dword_to_lds(a.bt + (int64_t)s * a.max_pages + lp, lds_address(id_lds) + (win & 1) * (kIdWindow * 4));
    };
    auto pages_of = [&](int tk, int tv, Pages& pg) {
        if constexpr (kLdsIds) {
            pg.k = id_lds[(tk * 4 + kpg) & (2 * kIdWindow - 1)];
            pg.v = id_lds[(tv * 4 + v_page) & (2 * kIdWindow - 1)];      // uniform; made scalar where it is used
        } else {
            pages_scalar(tk, tv, pg);
        }
    };
    // K(tk): instruction i of wave w moves chunk c = kPer*w + i of all 64 keys: four 256-byte runs, one per page.
    auto request_k = [&](int tk, int mine) {
        const unsigned char* src = (const unsigned char*)kpool + ((int64_t)mine * hkv + g) * (int64_t)(D * PS * 2) +
                                   (wu * kPer) * 256 + kslot * 16;
        const unsigned dst = lds_address(k_lds) + (tk % kKStages) * kTile + (wu * kPer) * 1024;
#pragma unroll
        for (int i = 0; i < kPer; ++i) load_to_lds(src + i * 256, dst + i * 1024);
    };
    // V(tv): a page's [half][channel][8 keys] layout is the LDS layout, so a V tile is sixteen 1 KiB runs;
    // wave w moves runs kPer*w .. kPer*w + kPer - 1, all of page v_page.
    constexpr int v_runs_per_page = 4;
    auto request_v = [&](int stage, int pid_any_lane) {
        const int pid = __builtin_amdgcn_readfirstlane(pid_any_lane);
        const unsigned char* src = (const unsigned char*)vpool + ((int64_t)pid * hkv + g) * (int64_t)(D * PS * 2) +
                                   ((wu * kPer) % v_runs_per_page) * 1024 + lane * 16;
        const unsigned dst = lds_address(v_lds) + stage * kTile + (wu * kPer) * 1024;
#pragma unroll
        for (int i = 0; i < kPer; ++i) load_to_lds(src + i * 1024, dst + i * 1024);
    };
    // Slots of the session's last page that hold no token may contain anything (NaN included) and would poison
    // the value product even under a zero weight: once V(tv) has landed, zero them in LDS.
    auto scrub_v = [&](int stage, int tv) {
        const int keep = ctx - (tv * BN + v_page * PS);         // slots < keep of this wave's page hold tokens
        if (keep < PS) {                                        // uniform over the wave
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int run = (wu * kPer) % v_runs_per_page + i;      // run = 2 * half + (channels 64..127)
                const int half = run >> 1;
                u32x4* p = reinterpret_cast<u32x4*>(v_lds + stage * kTile + (wu * kPer + i) * 1024 + lane * 16);
                *p = keep_quads(*p, keep - half * 4, keep - 8 - half * 4);
            }
        }
    };

    const float sl2 = a.scale * kLog2e;
    const int qpos = P + q0 + qrow0 + n;            // logical position of this lane's query
    float m = -INFINITY, lsum = 0.f;
    f32x16 o[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mb][i] = 0.f;

    const unsigned char* const k_lane = k_lds + n * 16 + hi * 1024;
    const unsigned char* const v_lane = v_lds + n * 16 + hi * 2048;

    // ---- prologue: K(0), K(1) requested and landed (and the first window of page ids) ----
    Pages pg;
    if constexpr (kLdsIds) {
        if (wu == 0) refill_ids(0);
    }
    pages_scalar(0, 0, pg);
    request_k(0, pg.k);
    pages_scalar(min(1, n_tiles - 1), 0, pg);
    request_k(1, pg.k);
    if (kVLead) {                                    // V(0) too when iteration t requests V(t + 1)
        pages_scalar(0, 0, pg);
        request_v(0, pg.v);
    }
    pages_scalar(min(2, n_tiles - 1), min(kVLead, n_tiles - 1), pg);   // what iteration 0 requests: V(kVLead) and K(2)
    AG_WAIT_VMCNT(0);
    __syncthreads();
    f32x16 sc[2];
    bf16x8 pa[4], pb[4];

    // Iteration t of a wave: S(t) from K(t) (matrix); then P(t) = exp2(S(t) - m) (vector) side by side with
    // O += V(t-1).P(t-1) (matrix).  At its start it requests V(t) and then K(t+2); at its end it waits until only
    // its own K(t+2) loads (and, with three V stages, V(t+1)) are outstanding, i.e. V(t) and K(t+1) have landed.
    // Requests are unconditional (past the last tile they repeat it into a buffer nobody reads), so the loop body has one
    // shape.  Every wave runs all n_tiles + 1 iterations (the barriers are workgroup-wide); the pieces a wave
    // does not need are skipped.
    auto iter = [&](int t, bf16x8 (&p_prev)[4], bf16x8 (&p_cur)[4]) {
        const int tv = min(t, n_tiles - 1);          // the V tile that must have landed when this iteration ends
        if constexpr (kLdsIds) {
            // The window holding tile t + 4 comes in one iteration before its first id is read (iteration t + 1
            // reads those of K(t + 4)); issued ahead of this iteration's tile requests, it has landed when wave 0
            // passes the wait at the end of the iteration, and the barrier there shows it to the other waves.
            // The slot it replaces holds the window two back, which nothing reads any more.
            if (wu == 0 && ((t + 4) & 15) == 0) refill_ids((t + 4) >> 4);
        }
        request_v((t + kVLead) % kVStages, pg.v);
        request_k(t + 2, pg.k);
        Pages nxt;                                    // ids for the next iteration's requests
        pages_of(min(t + 3, n_tiles - 1), min(t + 1 + kVLead, n_tiles - 1), nxt);
        const bool do_sm = t < wave_tiles, do_pv = t >= 1 && t <= wave_tiles;
        const unsigned char* kb = k_lane + (t % kKStages) * kTile;
        const unsigned char* vb = v_lane + ((t + kVStages - 1) % kVStages) * kTile;   // V(t-1)
        if (do_sm) {
            qk_tile(kb, qf, sc);
            if (t >= first_masked) {                 // the tile straddles this wave's diagonal
                const int kbase = t * BN + hi * 4;
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kbase + b * 32 + (i >> 2) * 8 + (i & 3);
                        sc[b][i] = key <= qpos ? sc[b][i] : -INFINITY;
                    }
            }
        }
        softmax_and_value_product(do_sm, do_pv, vb, sc, sl2, m, lsum, p_prev, p_cur, o);
        AG_WAIT_VMCNT(kPer * (1 + kVLead));
        scrub_v(t % kVStages, tv);
        pg = nxt;
        __syncthreads();
    };

#pragma unroll 1
    for (int t = 0; t <= n_tiles; t += 2) {
        iter(t, pb, pa);
        if (t + 1 <= n_tiles) iter(t + 1, pa, pb);
    }

    // ---- normalise, transpose through LDS, store rows contiguously ----
    AG_WAIT_VMCNT(0);                                // the last (redundant) tile requests still write to LDS
    __syncthreads();
    lsum += __shfl_xor(lsum, 32);
    const float inv = 1.0f / lsum;
    unsigned char* ob = lds + w * (32 * 256);       // this wave's [32 rows][128 ch] bf16, rows XOR-swizzled
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

template <int NW, int GP>
static ag_status launch_prefill_nw(const AttnArgs& a, hipStream_t st)
{
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load()) {
        ag_status e = hip_check(hipFuncSetAttribute((const void*)prefill_mfma_kernel<NW, GP>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(NW)),
                                "hipFuncSetAttribute(prefill)");
        if (e) return e;
        attr_set.store(true);
    }
    constexpr int BM = 32 * NW / GP;
    // sum_s ceil(N_s / BM) <= total_new / BM + batch, and no session has more than ceil(max_new / BM)
    const int64_t tiles_max = std::min<int64_t>((int64_t)a.total_rows / BM + a.batch,
                                                (int64_t)a.batch * ((a.max_new + BM - 1) / BM));
    const int64_t total = (GP == 1 ? a.hq : a.c.hkv) * tiles_max;
    const int64_t per_xcd = (total + 7) / 8;
    if (per_xcd * 8 > 0x7fffffff) { set_error("too many query tiles for one launch"); return AG_ERR_INVALID_ARG; }
    prof_before(st);
    hipLaunchKernelGGL((prefill_mfma_kernel<NW, GP>), dim3((unsigned)(per_xcd * 8)), dim3(64 * NW), lds_bytes(NW), st, a,
                       (int)tiles_max, (int)per_xcd, total);
    prof_after(st);
    return hip_check(hipGetLastError(), "prefill launch");
}

ag_status launch_prefill_mfma(const AttnArgs& a, hipStream_t st)
{
    const int G = a.hq / a.c.hkv;
    // 256-row workgroups when chunks are long enough to fill them (a K/V tile then feeds twice the rows);
    // 128-row workgroups keep short, ragged chunks efficient.  Groups of 2, 4 or 8 query heads share a workgroup
    // (a group of 8 only fits the 256-row form).
    const bool big = a.max_new >= 512;
    if (G == 4) return big ? launch_prefill_nw<8, 4>(a, st) : launch_prefill_nw<4, 4>(a, st);
    if (G == 2) return big ? launch_prefill_nw<8, 2>(a, st) : launch_prefill_nw<4, 2>(a, st);
    if (G == 8) return launch_prefill_nw<8, 8>(a, st);
    return big ? launch_prefill_nw<8, 1>(a, st) : launch_prefill_nw<4, 1>(a, st);
}

}  // namespace ag
