// Internal declarations shared by the host entry points and the kernel files.
// Nothing here is part of the ABI (that is include/ag.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ag.h"

namespace ag {

// Element offset of (slot, channel) inside one (page, head) block of the value pool.  Page sizes of 16 and
// more are stored as chunks of 8 keys, [chunk][channel][8 keys]: chunk = 2 * (slot / 16) + ((slot / 4) & 1)
// and the position inside it is (slot & 3) + 4 * ((slot / 8) & 1), i.e. chunk 2g + h of a 16-slot group g
// holds slots h*4 + {0..3} and 8 + h*4 + {0..3}: the 8 keys one lane owns after the score product.  Smaller
// pages are plain [channel][slot].
__host__ __device__ inline int64_t v_offset(int slot, int ch, int ps, int d)
{
    if (ps < 16) return (int64_t)ch * ps + slot;
    const int chunk = ((slot >> 4) << 1) | ((slot >> 2) & 1);
    const int pos = (slot & 3) | (((slot >> 3) & 1) << 2);
    return ((int64_t)chunk * d + ch) * 8 + pos;
}

// Host-validated view of an ag_kv_cache.
struct CacheView {
    void* k;          // [num_pages][hkv][d/8][ps][8]
    void* v;          // [num_pages][hkv][ps/8][d][8], see v_offset
    int num_pages, ps, ps_shift, hkv, d, dtype;
};

// One attention problem as the kernels see it.  Prefill / resume rows are
// addressed through cu_new; a decode step has cu_new == nullptr and one row
// per session whose position is ctx_lens[s] - 1.
struct AttnArgs {
    const void* q;
    void* out;
    CacheView c;
    const int32_t* bt;
    int max_pages;
    const int32_t* prefix_lens;   // nullptr: all zero (cold prefill)
    const int32_t* new_lens;      // nullptr in decode
    const int32_t* cu_new;        // nullptr in decode
    const int32_t* ctx_lens;      // decode only
    int batch, total_rows, max_new, max_ctx, hq;
    float scale;
};

void set_error(const char* fmt, ...);
ag_status hip_check(hipError_t e, const char* what);

// Event bracket around a main-kernel launch; no-ops unless ag_prof_enable() is active on this thread.
void prof_before(hipStream_t st);
void prof_after(hipStream_t st);

// kernel launchers (each returns after enqueueing)
ag_status launch_kv_append(const CacheView& c, const void* k_new, const void* v_new, const int32_t* bt, int max_pages,
                           const int32_t* prefix_lens, const int32_t* new_lens, const int32_t* cu_new, int batch,
                           int total_new, hipStream_t st);
ag_status launch_attn_general(const AttnArgs& a, hipStream_t st);

// bf16, head_dim 128, page 16 matrix-core paths
bool      prefill_mfma_supported(const AttnArgs& a);
ag_status launch_prefill_mfma(const AttnArgs& a, hipStream_t st);
bool      decode_mfma_supported(const AttnArgs& a);
size_t    decode_workspace_bytes(int batch, int hq, int d, int max_ctx);
ag_status launch_decode_mfma(const AttnArgs& a, void* ws, hipStream_t st);
// the whole decode step (append + attention + merge) in one launch; same shapes as the matrix-core decode
size_t    decode_step_workspace_bytes(int batch, int hq, int d, int max_ctx);
ag_status launch_decode_step(const AttnArgs& a, const void* k_new, const void* v_new, void* ws, hipStream_t st);
// Address, on the current device, of the library's own decode workspace (AG_DECODE_STATIC_SCRATCH_BYTES bytes);
// looked up once per device, allocates nothing.
ag_status decode_static_scratch(void** ptr_out);

// merged decode + short-resume batch (same shapes as the decode path)
bool      merged_mfma_supported(const AttnArgs& a);
size_t    merged_workspace_bytes(int total_rows, int hq, int max_ctx);
ag_status launch_merged_mfma(const AttnArgs& a, void* ws, hipStream_t st);

ag_status launch_probe(uint32_t* ids_out, int n_wg, int spin_cycles, hipStream_t st);

// CUs of the current device, and the CUs the stream's launches may use (the bits of its CU mask; all of them
// for a stream without one).  Launchers that size a grid to the partition use these.
int device_cus();
int stream_cus(hipStream_t st);

}  // namespace ag
