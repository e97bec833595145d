/*
 * ag.h - C ABI of the paged-KV attention library for MI355X (gfx950).
 *
 * The library implements the GPU work behind the three request classes of an
 * agent-serving engine (paper Sec. I, Sec. II-A, Fig. 1):
 *   cold prefill   - causal attention over a whole prompt that also builds the
 *                    session's KV cache;
 *   resume prefill - an appended chunk (a tool's output) attends to the cached
 *                    prefix and causally to itself;
 *   short decode   - one query per session over its cached keys and values;
 * plus the KV append that builds the cache, and CU-masked streams, the AMD
 * counterpart of the paper's pre-created SM partitions (Sec. III-C), on which
 * prefill and decode kernels run side by side.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a comment says "host".
 *     The caller owns every buffer; the library allocates no device memory
 *     and keeps no state between calls (stream handles excepted).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; they never synchronise.
 *   - Return value is an ag_status.  Conditions the host can see (null
 *     pointers, unsupported shapes, bounds that contradict each other, a
 *     workspace that is too small) are reported BEFORE anything is enqueued.
 *     Device-resident data (page ids, lengths) is not validated: a page id
 *     outside [0, num_pages) or a length beyond the host-side bound is
 *     undefined behaviour, as for any paged-attention kernel.
 *     ag_last_error() returns a thread-local message for the last failure.
 *   - Layouts (row-major, innermost last):
 *       Q, O          [T][Hq][D]        token-major, sessions concatenated
 *       K_new, V_new  [T][Hkv][D]
 *       K pool        [num_pages][Hkv][D/8][page_size][8]   chunk-major: the 8
 *                     channels of chunk c of slot s sit at ((c * page_size) + s) * 8,
 *                     so the 16-byte pieces that neighbouring lanes fetch for
 *                     neighbouring tokens are contiguous
 *       V pool        [num_pages][Hkv][page_size/8][D][8]   transposed in chunks of
 *                     8 keys (the value product contracts over tokens, and the
 *                     matrix cores want the contracted index contiguous).  Within
 *                     each aligned group g of 16 slots, chunk 2g + h holds slots
 *                     h*4 + {0..3} and 8 + h*4 + {0..3}, in that order: the 8
 *                     keys a lane owns after the score product.  So slot s of
 *                     channel c sits at ((2*(s/16) + ((s/4)&1)) * D + c) * 8 +
 *                     (s&3) + 4*((s/8)&1).  Page sizes below 16 are stored as
 *                     plain [D][page_size].
 *       block_tables  int32 [B][max_pages_per_seq]; logical page p of session
 *                     s lives in physical page block_tables[s][p]
 *       cu_new        int32 [B+1], cu_new[0] = 0, cu_new[s+1]-cu_new[s] = new_lens[s]
 *   - Logical position j of a session is page j / page_size, slot j % page_size.
 *   - GQA: query head h reads KV head h / (Hq / Hkv).
 *   - Ordering (paper Sec. III-C, memory management: a decode must never see
 *     partly written KV): attention reads keys and values ONLY from the
 *     pools, so the ag_kv_append that writes a token must precede, on the
 *     same stream or through an event, any attention call that covers it.
 *   - Supported: dtype AG_F32 or AG_BF16; head_dim a multiple of 8, <= 256;
 *     page_size a power of two in [1, 256].  bf16 with head_dim 128 and page_size 16
 *     runs on the matrix-core kernels; every other supported combination
 *     runs on the general fp32-arithmetic kernels.
 */
#ifndef AG_H
#define AG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AG_API __attribute__((visibility("default")))

typedef enum {
    AG_OK = 0,
    AG_ERR_INVALID_ARG = -1,   /* null pointer, negative size, contradictory bounds */
    AG_ERR_UNSUPPORTED = -2,   /* dtype / head_dim / page_size outside the supported set */
    AG_ERR_WORKSPACE = -3,     /* decode workspace smaller than ag_attn_decode_workspace_bytes() */
    AG_ERR_HIP = -4,           /* a HIP runtime call failed; text in ag_last_error() */
    AG_ERR_NO_SPACE = -5       /* page manager (ag_pager.h): not enough free pages, sessions or row capacity */
} ag_status;

typedef enum { AG_F32 = 0, AG_BF16 = 1 } ag_dtype;

/* Describes caller-owned device memory; plain data, read during the call only. */
typedef struct {
    void*   k_pool;            /* device, [num_pages][num_kv_heads][head_dim/8][page_size][8] */
    void*   v_pool;            /* device, [num_pages][num_kv_heads][page_size/8][head_dim][8], see above */
    int32_t num_pages;
    int32_t page_size;
    int32_t num_kv_heads;
    int32_t head_dim;
    int32_t dtype;             /* ag_dtype */
} ag_kv_cache;

/*
 * KV append: the cache-building half of a prefill and the one token a decode
 * step adds (paper Sec. II-A: the prefill "builds the KV cache"; Sec. III-C:
 * the cache is shared by the prefill and decode sides).
 * New token i of session s (row cu_new[s] + i of k_new / v_new) is written to
 * logical position prefix_lens[s] + i for every KV head.  Bit-exact copy.
 * total_new = cu_new[batch] is the host-side bound that sizes the launch.
 * Two sessions appending to the same physical page is a caller error.
 * k_new, v_new and both pools must be 16-byte aligned.
 */
AG_API ag_status ag_kv_append(const ag_kv_cache* cache,
                       const void* k_new, const void* v_new,             /* device [T][Hkv][D] */
                       const int32_t* block_tables, int32_t max_pages_per_seq,
                       const int32_t* prefix_lens, const int32_t* new_lens,   /* device [B] */
                       const int32_t* cu_new,                                 /* device [B+1] */
                       int32_t batch, int32_t total_new, void* stream);

/*
 * Cold prefill (paper Sec. I, Sec. II-A): causal softmax attention of each
 * session's N_s = new_lens[s] tokens over themselves, keys and values read
 * back from the pages ag_kv_append has just written (prefix length 0):
 *   O[t,h,:] = softmax_j<=i( scale * Q[t,h,:].K(s,h/G,j) ) . V(s,h/G,j),  t = cu_new[s] + i.
 * max_new >= max_s new_lens[s] (host-side bound).  Sessions with N_s = 0
 * contribute no rows.
 */
AG_API ag_status ag_attn_prefill(const ag_kv_cache* cache, const void* q, void* out,   /* device [T][Hq][D] */
                          const int32_t* block_tables, int32_t max_pages_per_seq,
                          const int32_t* new_lens, const int32_t* cu_new,
                          int32_t batch, int32_t total_new, int32_t max_new,
                          int32_t num_q_heads, float scale, void* stream);

/*
 * Resume prefill (paper Sec. I: later prefills append tool output to the
 * cached context; Sec. II-A: prefix caching): row i of session s sits at
 * logical position P_s + i, P_s = prefix_lens[s], and sees keys 0 .. P_s + i:
 * the whole cached prefix plus the chunk up to itself.  The chunk's own K/V
 * must already be appended.  With every P_s = 0 this is ag_attn_prefill.
 * max_ctx >= max_s (P_s + N_s), and max_ctx <= max_pages_per_seq * page_size.
 */
AG_API ag_status ag_attn_resume(const ag_kv_cache* cache, const void* q, void* out,    /* device [T][Hq][D] */
                         const int32_t* block_tables, int32_t max_pages_per_seq,
                         const int32_t* prefix_lens, const int32_t* new_lens, const int32_t* cu_new,
                         int32_t batch, int32_t total_new, int32_t max_new, int32_t max_ctx,
                         int32_t num_q_heads, float scale, void* stream);

/*
 * Short decode (paper Sec. II-A; Sec. III-B "decode steps": each active
 * stream produces one token per step): one query per session over all
 * ctx_lens[s] cached positions.  ctx_lens[s] COUNTS the step's own token,
 * whose K/V must already be appended, so there is no mask and the result
 * equals the last row of a prefill over the same ctx_lens[s] tokens.
 * ctx_lens[s] = 0 gives a row of zeros.
 * The batch's (session, KV head) contexts are laid end to end and cut into
 * equal shares, one per workgroup (a share may end one context and start
 * the next); their partial (max, sum, weighted values) triples go through
 * `workspace`, whose previous contents do not matter, and are merged in a
 * fixed order, so results are reproducible.
 * workspace_bytes >= ag_attn_decode_workspace_bytes(batch, num_q_heads, head_dim, max_ctx),
 * 16-byte aligned.  Calls sharing a workspace must be ordered on one stream.
 * batch * num_kv_heads * ceil(max_ctx / 32) may not exceed 2^30 (AG_ERR_INVALID_ARG).
 */
AG_API size_t    ag_attn_decode_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t head_dim, int32_t max_ctx);
AG_API ag_status ag_attn_decode(const ag_kv_cache* cache, const void* q, void* out,    /* device [B][Hq][D] */
                         const int32_t* block_tables, int32_t max_pages_per_seq,
                         const int32_t* ctx_lens,                               /* device [B] */
                         int32_t batch, int32_t max_ctx,
                         int32_t num_q_heads, float scale,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * ag_attn_decode for callers that cannot allocate device memory or pass a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results, but the partials go through an array of AG_DECODE_STATIC_SCRATCH_BYTES bytes that is
 * part of the library's device image (one copy on every GPU the library runs on, held until the process
 * ends).  The call allocates and frees nothing; its first use on a device looks the array's address up once.
 * A step whose ag_attn_decode_workspace_bytes() exceeds AG_DECODE_STATIC_SCRATCH_BYTES is refused with
 * AG_ERR_WORKSPACE before anything is enqueued (config-2-sized steps - 64 sessions, 32 query heads, contexts
 * to 4096 - need 18.1 MB).  Nothing in the array has to start at zero and nothing is kept between calls, but
 * every call on a GPU uses that GPU's one array: calls that overlap on one GPU (different streams, no event
 * between them) race; order them on one stream or with events.
 */
#define AG_DECODE_STATIC_SCRATCH_BYTES (32u << 20)
AG_API ag_status ag_attn_decode_static(const ag_kv_cache* cache, const void* q, void* out,    /* device [B][Hq][D] */
                                const int32_t* block_tables, int32_t max_pages_per_seq,
                                const int32_t* ctx_lens,                               /* device [B] */
                                int32_t batch, int32_t max_ctx,
                                int32_t num_q_heads, float scale, void* stream);

/*
 * One decode step in one launch (paper Sec. III-B: every active stream produces one token per decode step;
 * Sec. II-A: the step first extends the cache by that token, then attends over it): for every session s the
 * step's token - row s of k_new / v_new, [B][Hkv][D] - is written to logical position ctx_lens[s] - 1 exactly as
 * ag_kv_append would write it, and the query of row s attends to all ctx_lens[s] positions exactly as
 * ag_attn_decode would: pools and output are bit-identical to those two calls one after the other.  What
 * differs is the schedule: the workgroup whose share of the batch ends a (session, KV head) context appends
 * its token before reading that page, and the workgroup that is last to finish a context's segments (an
 * atomic count per context) merges them, always in segment order.  ctx_lens[s] = 0: nothing is appended for s
 * and its output row is zeros.  Sessions must not share the page a token is appended to (as for ag_kv_append).
 * Supported shapes: bf16, head_dim 128, page_size 16, Hq / Hkv <= 16 (AG_ERR_UNSUPPORTED otherwise: use the two
 * calls).  k_new, v_new, q and the pools 16-byte aligned.
 * Workspace: at least ag_decode_step_workspace_bytes() bytes, 16-byte aligned.  Its first
 * AG_DECODE_STEP_COUNTER_BYTES bytes are the counters (one per session and KV head: batch * Hkv may not exceed
 * AG_DECODE_STEP_COUNTER_BYTES / 4, AG_ERR_INVALID_ARG otherwise): they must be ZERO before the first call
 * that uses the workspace (zero-fill it once after allocating it); every call leaves them zero, so later calls
 * - of any batch, head count or context bound the workspace is large enough for - need no clearing.  The rest
 * may hold anything.  Calls sharing a workspace must be ordered on one stream.  A call that does not run to
 * its end (device reset) leaves the counters undefined: clear them again.
 */
#define AG_DECODE_STEP_COUNTER_BYTES (256u << 10)
AG_API size_t    ag_decode_step_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t head_dim, int32_t max_ctx);
AG_API ag_status ag_decode_step(const ag_kv_cache* cache, const void* k_new, const void* v_new,   /* device [B][Hkv][D] */
                         const void* q, void* out,                               /* device [B][Hq][D] */
                         const int32_t* block_tables, int32_t max_pages_per_seq,
                         const int32_t* ctx_lens,                                /* device [B] */
                         int32_t batch, int32_t max_ctx, int32_t num_q_heads, float scale,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * The decode queue's batch in one launch (paper Sec. III-A: short resume prefills are merged with decodes;
 * Algorithm 1: a request joins Q_D if it is a decode or no longer than B_prefill).  Semantics are exactly
 * ag_attn_resume's: session s brings new_lens[s] >= 0 query rows at positions prefix_lens[s] + i that attend
 * causally to the session's keys; a decode is the case new_lens[s] = 1, prefix_lens[s] = ctx - 1.  What
 * differs is the schedule: the keys of the batch are dealt to the workgroups in equal shares as in
 * ag_attn_decode (streaming work for decodes and chunks of a few rows, tile work for longer chunks, side by
 * side), which pays when sessions bring few rows (the launch is then bound by reading K and V); when the
 * longest chunk (max_new) has 144 rows or more the call runs ag_attn_resume's kernel instead, which is faster
 * from about there on.  The launch is sized for the CUs `stream` may use (its CU mask, if it has one).
 * Arguments as ag_attn_resume, plus a device workspace of at least
 * ag_attn_merged_workspace_bytes(total_new, num_q_heads, max_ctx) bytes, 16-byte aligned, which the call may
 * overwrite entirely (AG_ERR_WORKSPACE if smaller).  Calls sharing a workspace must be ordered on one stream.
 */
AG_API size_t ag_attn_merged_workspace_bytes(int32_t total_new, int32_t num_q_heads, int32_t max_ctx);
AG_API ag_status ag_attn_merged(const ag_kv_cache* cache, const void* q, void* out,
                         const int32_t* block_tables, int32_t max_pages_per_seq,
                         const int32_t* prefix_lens, const int32_t* new_lens, const int32_t* cu_new, /* device */
                         int32_t batch, int32_t total_new, int32_t max_new, int32_t max_ctx,
                         int32_t num_q_heads, float scale,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * CU-masked streams: the counterpart of the paper's pre-created SM partitions
 * (Sec. III-C; Algorithm 1 "partition SMs").  Kernels launched on the returned
 * stream run only on the compute units whose bit is set.  cu_mask_words is a
 * HOST array of n_words 32-bit words, bit b of word w = mask bit 32*w + b, in
 * the order the HIP runtime defines for hipExtStreamCreateWithCUMask; at least
 * one bit must be set.  The stream has default priority.  Destroy with
 * ag_stream_destroy.  *stream_out is a hipStream_t.
 */
AG_API ag_status ag_stream_create_cumask(void** stream_out, const uint32_t* cu_mask_words, int32_t n_words);
AG_API ag_status ag_stream_destroy(void* stream);

/*
 * Builds mask words (host) that select the same CUs in every XCD, so that a
 * partition never empties one XCD: workgroups are dealt to XCDs round-robin,
 * and mask bit b addresses XCD b % n_xcd, CU b / n_xcd of that XCD.  Sets the
 * bits of CUs [first_cu_per_xcd, first_cu_per_xcd + cus_per_xcd) of each XCD;
 * total_cus = n_xcd * (CUs per XCD).  Paper Eq. for the discrete allocation
 * set {g, 2g, ..., S}: here g = n_xcd CUs.  On MI355X CU k of an XCD sits in
 * shader engine k % 4, and workgroups are dealt evenly to the engines that have
 * a CU enabled: a count that is not a multiple of 4 leaves the engines uneven
 * and runs like the next lower multiple (6 CUs per XCD measure like 4), so 4
 * CUs per XCD (32 CUs) is the useful step.
 */
AG_API ag_status ag_cumask_build(uint32_t* words, int32_t n_words, int32_t total_cus, int32_t n_xcd,
                          int32_t first_cu_per_xcd, int32_t cus_per_xcd);

/*
 * Measurement aid for the partition: launches n_workgroups one-wave
 * workgroups on `stream`; each spins for about `spin_cycles` clock ticks so
 * that the launch spreads over every CU the stream may use, then records
 * where it ran.  ids_out (device, n_workgroups uint32): bits 0-7 the CU id
 * within its shader array, 8-11 shader array, 12-15 shader engine, 16-19 XCD.
 */
AG_API ag_status ag_probe_placement(uint32_t* ids_out, int32_t n_workgroups, int32_t spin_cycles, void* stream);

/* Device facts (host out-pointers, any may be NULL): CU count, XCD count if the runtime reports it else 0. */
AG_API ag_status ag_device_info(int32_t* num_cus, int32_t* num_xcd, int32_t* wavefront_size, char* arch_name, int32_t arch_name_len);

/*
 * Synchronous checker for tests: copies the device-resident block tables and
 * lengths to the host and verifies what the fast path assumes (page ids in
 * range for every logical page in use, lengths within max_pages_per_seq *
 * page_size, cu_new consistent).  prefix_lens or cu_new may be NULL.
 * Synchronises `stream`.  Returns AG_ERR_INVALID_ARG with a message on the
 * first violation.
 */
AG_API ag_status ag_debug_validate(const ag_kv_cache* cache, const int32_t* block_tables, int32_t max_pages_per_seq,
                            const int32_t* prefix_lens, const int32_t* new_lens, const int32_t* cu_new,
                            int32_t batch, void* stream);

/*
 * Measurement aid, not part of the serving path.  While enabled on the calling
 * host thread, every attention call's main kernel work (both kernels of
 * ag_attn_decode, split and merge; the one kernel of ag_decode_step; the tile
 * kernel of ag_attn_prefill / ag_attn_resume; the split kernel of
 * ag_attn_merged; or the general kernel) is bracketed by a pair of HIP events
 * recorded on the launch stream, up to max_launches pairs.  ag_prof_collect
 * waits for the recorded events, returns the mean / min / max duration of
 * those launches in microseconds (any out-pointer may be NULL) and starts a
 * new series.  ag_prof_disable releases the events.  Host objects only; no
 * device memory is allocated.
 */
AG_API ag_status ag_prof_enable(int32_t max_launches);
AG_API ag_status ag_prof_collect(double* mean_us, double* min_us, double* max_us, int32_t* n_launches);
AG_API ag_status ag_prof_disable(void);

AG_API const char* ag_status_string(ag_status s);
AG_API const char* ag_last_error(void);       /* thread-local; valid until the next failing call on this thread */
AG_API const char* ag_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AG_H */
