// C-ABI entry points: argument validation and launch planning.  Every check a
// host can make happens here, before anything is enqueued (see include/ag.h).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "ag_internal.h"

namespace ag {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

ag_status hip_check(hipError_t e, const char* what)
{
    if (e == hipSuccess) return AG_OK;
    set_error("%s: %s", what, hipGetErrorString(e));
    return AG_ERR_HIP;
}

struct Prof {
    bool on = false;
    int cap = 0, n = 0;
    bool open = false;
    std::vector<hipEvent_t> ev;      // 2 per launch: start, stop
};
static thread_local Prof g_prof;

void prof_before(hipStream_t st)
{
    Prof& p = g_prof;
    if (!p.on || p.n >= p.cap) return;
    p.open = hipEventRecord(p.ev[2 * p.n], st) == hipSuccess;
}

void prof_after(hipStream_t st)
{
    Prof& p = g_prof;
    if (!p.on || !p.open) return;
    p.open = false;
    if (hipEventRecord(p.ev[2 * p.n + 1], st) == hipSuccess) ++p.n;
}

static int log2_exact(int x)
{
    if (x <= 0 || (x & (x - 1))) return -1;
    int s = 0;
    while ((1 << s) < x) ++s;
    return s;
}

static ag_status view_cache(const ag_kv_cache* c, CacheView* v)
{
    if (!c) { set_error("cache is NULL"); return AG_ERR_INVALID_ARG; }
    if (!c->k_pool || !c->v_pool) { set_error("cache pools are NULL"); return AG_ERR_INVALID_ARG; }
    if (c->num_pages <= 0 || c->num_kv_heads <= 0) {
        set_error("num_pages=%d num_kv_heads=%d must be positive", c->num_pages, c->num_kv_heads);
        return AG_ERR_INVALID_ARG;
    }
    if (c->dtype != AG_F32 && c->dtype != AG_BF16) { set_error("dtype %d unsupported", c->dtype); return AG_ERR_UNSUPPORTED; }
    if (c->head_dim <= 0 || c->head_dim > 256 || c->head_dim % 8) {
        set_error("head_dim %d unsupported (multiple of 8, at most 256)", c->head_dim);
        return AG_ERR_UNSUPPORTED;
    }
    const int sh = log2_exact(c->page_size);
    if (sh < 0 || c->page_size > 256) {
        set_error("page_size %d unsupported (power of two, at most 256)", c->page_size);
        return AG_ERR_UNSUPPORTED;
    }
    v->k = c->k_pool; v->v = c->v_pool;
    v->num_pages = c->num_pages; v->ps = c->page_size; v->ps_shift = sh;
    v->hkv = c->num_kv_heads; v->d = c->head_dim; v->dtype = c->dtype;
    return AG_OK;
}

static ag_status check_heads(const CacheView& c, int hq)
{
    if (hq <= 0 || hq % c.hkv) {
        set_error("num_q_heads %d is not a positive multiple of num_kv_heads %d", hq, c.hkv);
        return AG_ERR_INVALID_ARG;
    }
    return AG_OK;
}

static ag_status check_scale(float scale)
{
    if (!(scale > 0.0f) || !(scale < 1e30f)) { set_error("scale must be positive and finite"); return AG_ERR_INVALID_ARG; }
    return AG_OK;
}

static ag_status prefill_common(const ag_kv_cache* cache, const void* q, void* out, const int32_t* bt, int max_pages,
                                const int32_t* prefix_lens, bool need_prefix, const int32_t* new_lens,
                                const int32_t* cu_new, int batch, int total_new, int max_new, int max_ctx, int hq,
                                float scale, void* stream, bool merged = false, void* workspace = nullptr,
                                size_t workspace_bytes = 0)
{
    CacheView c;
    ag_status st = view_cache(cache, &c);
    if (st) return st;
    if (!q || !out || !bt || !new_lens || !cu_new || (need_prefix && !prefix_lens)) {
        set_error("a required pointer is NULL");
        return AG_ERR_INVALID_ARG;
    }
    if (batch <= 0 || max_pages <= 0 || total_new < 0 || max_new < 0) {
        set_error("batch=%d max_pages_per_seq=%d total_new=%d max_new=%d: sizes must be positive", batch, max_pages,
                  total_new, max_new);
        return AG_ERR_INVALID_ARG;
    }
    if ((st = check_heads(c, hq)) || (st = check_scale(scale))) return st;
    if (max_new > total_new) { set_error("max_new %d exceeds total_new %d", max_new, total_new); return AG_ERR_INVALID_ARG; }
    if (max_ctx < max_new) { set_error("max_ctx %d is smaller than max_new %d", max_ctx, max_new); return AG_ERR_INVALID_ARG; }
    if ((int64_t)max_ctx > (int64_t)max_pages * c.ps) {
        set_error("max_ctx %d exceeds max_pages_per_seq * page_size = %lld", max_ctx, (long long)max_pages * c.ps);
        return AG_ERR_INVALID_ARG;
    }
    if (merged) {
        const size_t need = merged_workspace_bytes(total_new, hq, max_ctx);
        if (workspace_bytes < need || (need && !workspace)) {
            set_error("merged-batch workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
            return AG_ERR_WORKSPACE;
        }
        if (((uintptr_t)workspace) % 16) { set_error("merged-batch workspace must be 16-byte aligned"); return AG_ERR_INVALID_ARG; }
    }
    if (total_new == 0 || max_new == 0) return AG_OK;

    AttnArgs a;
    a.q = q; a.out = out; a.c = c; a.bt = bt; a.max_pages = max_pages;
    a.prefix_lens = prefix_lens; a.new_lens = new_lens; a.cu_new = cu_new; a.ctx_lens = nullptr;
    a.batch = batch; a.total_rows = total_new; a.max_new = max_new; a.max_ctx = max_ctx; a.hq = hq; a.scale = scale;
    if (merged) {
        // The merged kernel cuts a chunk into items of 32 rows (at G = 4), each of which walks the chunk's whole
        // prefix; once chunks are long the prefill kernel's larger tiles are faster even with the decodes in the
        // same launch (64 decodes + 8 chunks on 2-8k-token prefixes: 237 against 248 us at 128 rows per chunk, 294
        // against 268 us at 192), and the semantics are the same.
        constexpr int kMergedRowsLimit = 144;
        if (max_new >= kMergedRowsLimit && prefill_mfma_supported(a)) return launch_prefill_mfma(a, (hipStream_t)stream);
        if (merged_mfma_supported(a)) return launch_merged_mfma(a, workspace, (hipStream_t)stream);
        return launch_attn_general(a, (hipStream_t)stream);
    }
    if (prefill_mfma_supported(a)) return launch_prefill_mfma(a, (hipStream_t)stream);
    return launch_attn_general(a, (hipStream_t)stream);
}

}  // namespace ag

using namespace ag;

extern "C" {

ag_status ag_kv_append(const ag_kv_cache* cache, const void* k_new, const void* v_new, const int32_t* block_tables,
                       int32_t max_pages_per_seq, const int32_t* prefix_lens, const int32_t* new_lens,
                       const int32_t* cu_new, int32_t batch, int32_t total_new, void* stream)
{
    CacheView c;
    ag_status st = view_cache(cache, &c);
    if (st) return st;
    if (!k_new || !v_new || !block_tables || !prefix_lens || !new_lens || !cu_new) {
        set_error("a required pointer is NULL");
        return AG_ERR_INVALID_ARG;
    }
    if (batch <= 0 || max_pages_per_seq <= 0 || total_new < 0) {
        set_error("batch=%d max_pages_per_seq=%d total_new=%d: sizes must be positive", batch, max_pages_per_seq, total_new);
        return AG_ERR_INVALID_ARG;
    }
    if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)c.k | (uintptr_t)c.v) % 16) {
        set_error("k_new, v_new and the pools must be 16-byte aligned");
        return AG_ERR_INVALID_ARG;
    }
    if (total_new == 0) return AG_OK;
    return launch_kv_append(c, k_new, v_new, block_tables, max_pages_per_seq, prefix_lens, new_lens, cu_new, batch,
                            total_new, (hipStream_t)stream);
}

ag_status ag_attn_prefill(const ag_kv_cache* cache, const void* q, void* out, const int32_t* block_tables,
                          int32_t max_pages_per_seq, const int32_t* new_lens, const int32_t* cu_new, int32_t batch,
                          int32_t total_new, int32_t max_new, int32_t num_q_heads, float scale, void* stream)
{
    return prefill_common(cache, q, out, block_tables, max_pages_per_seq, nullptr, false, new_lens, cu_new, batch,
                          total_new, max_new, max_new, num_q_heads, scale, stream);
}

ag_status ag_attn_resume(const ag_kv_cache* cache, const void* q, void* out, const int32_t* block_tables,
                         int32_t max_pages_per_seq, const int32_t* prefix_lens, const int32_t* new_lens,
                         const int32_t* cu_new, int32_t batch, int32_t total_new, int32_t max_new, int32_t max_ctx,
                         int32_t num_q_heads, float scale, void* stream)
{
    return prefill_common(cache, q, out, block_tables, max_pages_per_seq, prefix_lens, true, new_lens, cu_new, batch,
                          total_new, max_new, max_ctx, num_q_heads, scale, stream);
}

size_t ag_attn_merged_workspace_bytes(int32_t total_new, int32_t num_q_heads, int32_t max_ctx)
{
    if (total_new < 0 || num_q_heads <= 0 || max_ctx < 0) return 0;
    return merged_workspace_bytes(total_new, num_q_heads, max_ctx);
}

ag_status ag_attn_merged(const ag_kv_cache* cache, const void* q, void* out, const int32_t* block_tables,
                         int32_t max_pages_per_seq, const int32_t* prefix_lens, const int32_t* new_lens,
                         const int32_t* cu_new, int32_t batch, int32_t total_new, int32_t max_new, int32_t max_ctx,
                         int32_t num_q_heads, float scale, void* workspace, size_t workspace_bytes, void* stream)
{
    return prefill_common(cache, q, out, block_tables, max_pages_per_seq, prefix_lens, true, new_lens, cu_new, batch,
                          total_new, max_new, max_ctx, num_q_heads, scale, stream, true, workspace, workspace_bytes);
}

size_t ag_attn_decode_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t head_dim, int32_t max_ctx)
{
    if (batch <= 0 || num_q_heads <= 0 || head_dim <= 0 || max_ctx < 0) return 0;
    return decode_workspace_bytes(batch, num_q_heads, head_dim, max_ctx);
}

// Shared body of the two decode entry points.  own_scratch: the workspace is the library's static array
// (looked up only after every host-side check has passed) instead of the caller's.
static ag_status decode_common(const ag_kv_cache* cache, const void* q, void* out, const int32_t* block_tables,
                               int32_t max_pages_per_seq, const int32_t* ctx_lens, int32_t batch, int32_t max_ctx,
                               int32_t num_q_heads, float scale, void* workspace, size_t workspace_bytes,
                               bool own_scratch, void* stream)
{
    CacheView c;
    ag_status st = view_cache(cache, &c);
    if (st) return st;
    if (!q || !out || !block_tables || !ctx_lens) { set_error("a required pointer is NULL"); return AG_ERR_INVALID_ARG; }
    if (batch <= 0 || max_pages_per_seq <= 0 || max_ctx < 0) {
        set_error("batch=%d max_pages_per_seq=%d max_ctx=%d: sizes must be positive", batch, max_pages_per_seq, max_ctx);
        return AG_ERR_INVALID_ARG;
    }
    if ((st = check_heads(c, num_q_heads)) || (st = check_scale(scale))) return st;
    if ((int64_t)max_ctx > (int64_t)max_pages_per_seq * c.ps) {
        set_error("max_ctx %d exceeds max_pages_per_seq * page_size = %lld", max_ctx, (long long)max_pages_per_seq * c.ps);
        return AG_ERR_INVALID_ARG;
    }
    const size_t need = decode_workspace_bytes(batch, num_q_heads, c.d, max_ctx);
    if (own_scratch) {
        if (need > (size_t)AG_DECODE_STATIC_SCRATCH_BYTES) {
            set_error("decode step needs %zu bytes of workspace, the library's own scratch holds %zu: reduce batch * "
                      "num_q_heads * max_ctx or call ag_attn_decode with a workspace", need,
                      (size_t)AG_DECODE_STATIC_SCRATCH_BYTES);
            return AG_ERR_WORKSPACE;
        }
        if ((st = decode_static_scratch(&workspace))) return st;
    } else {
        if (workspace_bytes < need || (need && !workspace)) {
            set_error("decode workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
            return AG_ERR_WORKSPACE;
        }
        if (((uintptr_t)workspace) % 16) { set_error("decode workspace must be 16-byte aligned"); return AG_ERR_INVALID_ARG; }
    }

    AttnArgs a;
    a.q = q; a.out = out; a.c = c; a.bt = block_tables; a.max_pages = max_pages_per_seq;
    a.prefix_lens = nullptr; a.new_lens = nullptr; a.cu_new = nullptr; a.ctx_lens = ctx_lens;
    a.batch = batch; a.total_rows = batch; a.max_new = 1; a.max_ctx = max_ctx; a.hq = num_q_heads; a.scale = scale;
    if (decode_mfma_supported(a)) return launch_decode_mfma(a, workspace, (hipStream_t)stream);
    return launch_attn_general(a, (hipStream_t)stream);
}

ag_status ag_attn_decode(const ag_kv_cache* cache, const void* q, void* out, const int32_t* block_tables,
                         int32_t max_pages_per_seq, const int32_t* ctx_lens, int32_t batch, int32_t max_ctx,
                         int32_t num_q_heads, float scale, void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_common(cache, q, out, block_tables, max_pages_per_seq, ctx_lens, batch, max_ctx, num_q_heads, scale,
                         workspace, workspace_bytes, false, stream);
}

ag_status ag_attn_decode_static(const ag_kv_cache* cache, const void* q, void* out, const int32_t* block_tables,
                                int32_t max_pages_per_seq, const int32_t* ctx_lens, int32_t batch, int32_t max_ctx,
                                int32_t num_q_heads, float scale, void* stream)
{
    return decode_common(cache, q, out, block_tables, max_pages_per_seq, ctx_lens, batch, max_ctx, num_q_heads, scale,
                         nullptr, 0, true, stream);
}

size_t ag_decode_step_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t head_dim, int32_t max_ctx)
{
    if (batch <= 0 || num_q_heads <= 0 || head_dim <= 0 || max_ctx < 0) return 0;
    return decode_step_workspace_bytes(batch, num_q_heads, head_dim, max_ctx);
}

ag_status ag_decode_step(const ag_kv_cache* cache, const void* k_new, const void* v_new, const void* q, void* out,
                         const int32_t* block_tables, int32_t max_pages_per_seq, const int32_t* ctx_lens, int32_t batch,
                         int32_t max_ctx, int32_t num_q_heads, float scale, void* workspace, size_t workspace_bytes,
                         void* stream)
{
    CacheView c;
    ag_status st = view_cache(cache, &c);
    if (st) return st;
    if (!k_new || !v_new || !q || !out || !block_tables || !ctx_lens) { set_error("a required pointer is NULL"); return AG_ERR_INVALID_ARG; }
    if (batch <= 0 || max_pages_per_seq <= 0 || max_ctx < 0) {
        set_error("batch=%d max_pages_per_seq=%d max_ctx=%d: sizes must be positive", batch, max_pages_per_seq, max_ctx);
        return AG_ERR_INVALID_ARG;
    }
    if ((st = check_heads(c, num_q_heads)) || (st = check_scale(scale))) return st;
    if ((int64_t)max_ctx > (int64_t)max_pages_per_seq * c.ps) {
        set_error("max_ctx %d exceeds max_pages_per_seq * page_size = %lld", max_ctx, (long long)max_pages_per_seq * c.ps);
        return AG_ERR_INVALID_ARG;
    }
    if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)c.k | (uintptr_t)c.v) % 16) {
        set_error("k_new, v_new and the pools must be 16-byte aligned");
        return AG_ERR_INVALID_ARG;
    }
    AttnArgs a;
    a.q = q; a.out = out; a.c = c; a.bt = block_tables; a.max_pages = max_pages_per_seq;
    a.prefix_lens = nullptr; a.new_lens = nullptr; a.cu_new = nullptr; a.ctx_lens = ctx_lens;
    a.batch = batch; a.total_rows = batch; a.max_new = 1; a.max_ctx = max_ctx; a.hq = num_q_heads; a.scale = scale;
    if (!decode_mfma_supported(a)) {
        set_error("ag_decode_step covers bf16, head_dim 128, page_size 16, at most 16 query heads per KV head, 16-byte "
                  "aligned q; use ag_kv_append + ag_attn_decode for other shapes");
        return AG_ERR_UNSUPPORTED;
    }
    const size_t need = decode_step_workspace_bytes(batch, num_q_heads, c.d, max_ctx);
    if (workspace_bytes < need || !workspace) {
        set_error("decode-step workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
        return AG_ERR_WORKSPACE;
    }
    if (((uintptr_t)workspace) % 16) { set_error("decode-step workspace must be 16-byte aligned"); return AG_ERR_INVALID_ARG; }
    return launch_decode_step(a, k_new, v_new, workspace, (hipStream_t)stream);
}

ag_status ag_stream_create_cumask(void** stream_out, const uint32_t* cu_mask_words, int32_t n_words)
{
    if (!stream_out || !cu_mask_words || n_words <= 0 || n_words > 64) {
        set_error("stream_out / cu_mask_words NULL or n_words=%d out of range", n_words);
        return AG_ERR_INVALID_ARG;
    }
    uint32_t any = 0;
    for (int i = 0; i < n_words; ++i) any |= cu_mask_words[i];
    if (!any) { set_error("CU mask selects no compute unit"); return AG_ERR_INVALID_ARG; }
    hipStream_t s = nullptr;
    ag_status st = hip_check(hipExtStreamCreateWithCUMask(&s, (uint32_t)n_words, cu_mask_words), "hipExtStreamCreateWithCUMask");
    if (st) return st;
    *stream_out = (void*)s;
    return AG_OK;
}

ag_status ag_stream_destroy(void* stream)
{
    if (!stream) { set_error("stream is NULL"); return AG_ERR_INVALID_ARG; }
    return hip_check(hipStreamDestroy((hipStream_t)stream), "hipStreamDestroy");
}

ag_status ag_cumask_build(uint32_t* words, int32_t n_words, int32_t total_cus, int32_t n_xcd,
                          int32_t first_cu_per_xcd, int32_t cus_per_xcd)
{
    if (!words || n_words <= 0 || total_cus <= 0 || n_xcd <= 0 || total_cus % n_xcd) {
        set_error("words NULL, or total_cus=%d not a positive multiple of n_xcd=%d", total_cus, n_xcd);
        return AG_ERR_INVALID_ARG;
    }
    const int per = total_cus / n_xcd;
    if (first_cu_per_xcd < 0 || cus_per_xcd <= 0 || first_cu_per_xcd + cus_per_xcd > per) {
        set_error("CUs [%d, %d) do not fit an XCD of %d CUs", first_cu_per_xcd, first_cu_per_xcd + cus_per_xcd, per);
        return AG_ERR_INVALID_ARG;
    }
    if ((int64_t)n_words * 32 < total_cus) { set_error("%d words cannot hold %d mask bits", n_words, total_cus); return AG_ERR_INVALID_ARG; }
    memset(words, 0, sizeof(uint32_t) * (size_t)n_words);
    for (int cu = first_cu_per_xcd; cu < first_cu_per_xcd + cus_per_xcd; ++cu)
        for (int x = 0; x < n_xcd; ++x) {
            const int bit = cu * n_xcd + x;
            words[bit >> 5] |= 1u << (bit & 31);
        }
    return AG_OK;
}

ag_status ag_probe_placement(uint32_t* ids_out, int32_t n_workgroups, int32_t spin_cycles, void* stream)
{
    if (!ids_out || n_workgroups <= 0 || spin_cycles < 0 || spin_cycles > (1 << 26)) {
        set_error("ids_out NULL, n_workgroups=%d or spin_cycles=%d out of range", n_workgroups, spin_cycles);
        return AG_ERR_INVALID_ARG;
    }
    return launch_probe(ids_out, n_workgroups, spin_cycles, (hipStream_t)stream);
}

ag_status ag_device_info(int32_t* num_cus, int32_t* num_xcd, int32_t* wavefront_size, char* arch_name, int32_t arch_name_len)
{
    int dev = 0;
    ag_status st = hip_check(hipGetDevice(&dev), "hipGetDevice");
    if (st) return st;
    hipDeviceProp_t p;
    if ((st = hip_check(hipGetDeviceProperties(&p, dev), "hipGetDeviceProperties"))) return st;
    if (num_cus) *num_cus = p.multiProcessorCount;
    if (wavefront_size) *wavefront_size = p.warpSize;
    if (num_xcd) {
        int x = 0;
        if (hipDeviceGetAttribute(&x, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess) { (void)hipGetLastError(); x = 0; }
        *num_xcd = x;
    }
    if (arch_name && arch_name_len > 0) {
        strncpy(arch_name, p.gcnArchName, (size_t)arch_name_len - 1);
        arch_name[arch_name_len - 1] = 0;
    }
    return AG_OK;
}

ag_status ag_debug_validate(const ag_kv_cache* cache, const int32_t* block_tables, int32_t max_pages_per_seq,
                            const int32_t* prefix_lens, const int32_t* new_lens, const int32_t* cu_new, int32_t batch,
                            void* stream)
{
    CacheView c;
    ag_status st = view_cache(cache, &c);
    if (st) return st;
    if (!block_tables || !new_lens || batch <= 0 || max_pages_per_seq <= 0) {
        set_error("block_tables / new_lens NULL or sizes not positive");
        return AG_ERR_INVALID_ARG;
    }
    if ((st = hip_check(hipStreamSynchronize((hipStream_t)stream), "hipStreamSynchronize"))) return st;
    std::vector<int32_t> bt((size_t)batch * max_pages_per_seq), pl(batch, 0), nl(batch), cu(batch + 1, 0);
    if ((st = hip_check(hipMemcpy(bt.data(), block_tables, bt.size() * 4, hipMemcpyDeviceToHost), "copy block_tables"))) return st;
    if ((st = hip_check(hipMemcpy(nl.data(), new_lens, nl.size() * 4, hipMemcpyDeviceToHost), "copy new_lens"))) return st;
    if (prefix_lens && (st = hip_check(hipMemcpy(pl.data(), prefix_lens, pl.size() * 4, hipMemcpyDeviceToHost), "copy prefix_lens"))) return st;
    if (cu_new && (st = hip_check(hipMemcpy(cu.data(), cu_new, cu.size() * 4, hipMemcpyDeviceToHost), "copy cu_new"))) return st;
    int64_t run = 0;
    for (int s = 0; s < batch; ++s) {
        if (pl[s] < 0 || nl[s] < 0) { set_error("session %d: negative length", s); return AG_ERR_INVALID_ARG; }
        if (cu_new && cu[s] != run) { set_error("session %d: cu_new=%d, expected %lld", s, cu[s], (long long)run); return AG_ERR_INVALID_ARG; }
        run += nl[s];
        const int64_t ctx = (int64_t)pl[s] + nl[s];
        if (ctx > (int64_t)max_pages_per_seq * c.ps) {
            set_error("session %d: context %lld exceeds max_pages_per_seq * page_size", s, (long long)ctx);
            return AG_ERR_INVALID_ARG;
        }
        const int pages = (int)((ctx + c.ps - 1) >> c.ps_shift);
        for (int p = 0; p < pages; ++p) {
            const int32_t id = bt[(size_t)s * max_pages_per_seq + p];
            if (id < 0 || id >= c.num_pages) {
                set_error("session %d logical page %d: physical page %d outside [0, %d)", s, p, id, c.num_pages);
                return AG_ERR_INVALID_ARG;
            }
        }
    }
    if (cu_new && cu[batch] != run) { set_error("cu_new[batch]=%d, expected %lld", cu[batch], (long long)run); return AG_ERR_INVALID_ARG; }
    return AG_OK;
}

ag_status ag_prof_enable(int32_t max_launches)
{
    if (max_launches <= 0 || max_launches > (1 << 20)) { set_error("max_launches=%d out of range", max_launches); return AG_ERR_INVALID_ARG; }
    ag_prof_disable();
    Prof& p = g_prof;
    p.ev.resize(2 * (size_t)max_launches);
    for (size_t i = 0; i < p.ev.size(); ++i) {
        ag_status st = hip_check(hipEventCreate(&p.ev[i]), "hipEventCreate");
        if (st) { for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(p.ev[j]); p.ev.clear(); return st; }
    }
    p.cap = max_launches; p.n = 0; p.open = false; p.on = true;
    return AG_OK;
}

ag_status ag_prof_collect(double* mean_us, double* min_us, double* max_us, int32_t* n_launches)
{
    Prof& p = g_prof;
    if (!p.on) { set_error("profiling is not enabled on this thread"); return AG_ERR_INVALID_ARG; }
    double sum = 0, lo = 1e30, hi = 0;
    for (int i = 0; i < p.n; ++i) {
        ag_status st = hip_check(hipEventSynchronize(p.ev[2 * i + 1]), "hipEventSynchronize");
        if (st) return st;
        float ms = 0;
        if ((st = hip_check(hipEventElapsedTime(&ms, p.ev[2 * i], p.ev[2 * i + 1]), "hipEventElapsedTime"))) return st;
        const double us = 1e3 * ms;
        sum += us; lo = us < lo ? us : lo; hi = us > hi ? us : hi;
    }
    if (mean_us) *mean_us = p.n ? sum / p.n : 0.0;
    if (min_us) *min_us = p.n ? lo : 0.0;
    if (max_us) *max_us = hi;
    if (n_launches) *n_launches = p.n;
    p.n = 0; p.open = false;
    return AG_OK;
}

ag_status ag_prof_disable(void)
{
    Prof& p = g_prof;
    for (hipEvent_t e : p.ev) (void)hipEventDestroy(e);
    p.ev.clear();
    p.on = false; p.cap = 0; p.n = 0; p.open = false;
    return AG_OK;
}

const char* ag_status_string(ag_status s)
{
    switch (s) {
        case AG_OK: return "AG_OK";
        case AG_ERR_INVALID_ARG: return "AG_ERR_INVALID_ARG";
        case AG_ERR_UNSUPPORTED: return "AG_ERR_UNSUPPORTED";
        case AG_ERR_WORKSPACE: return "AG_ERR_WORKSPACE";
        case AG_ERR_HIP: return "AG_ERR_HIP";
        case AG_ERR_NO_SPACE: return "AG_ERR_NO_SPACE";
    }
    return "AG_ERR_UNKNOWN";
}

const char* ag_last_error(void) { return g_err; }

const char* ag_version(void) { return "agattn 0.1 (gfx950)"; }

}  // extern "C"
