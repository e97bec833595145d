// Internal declarations shared by the host entry points and the kernel files.
// Nothing here is part of the ABI (that is include/ag.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ag.h"

namespace ag {

// Column of slot s inside a value-page row: the two middle quads of every aligned 16 are swapped.
__host__ __device__ inline int v_col(int slot, int ps) { return ps < 16 ? slot : ((slot & ~12) | ((slot & 8) >> 1) | ((slot & 4) << 1)); }

// Host-validated view of an ag_kv_cache.
struct CacheView {
    void* k;          // [num_pages][hkv][d/8][ps][8]
    void* v;          // [num_pages][hkv][d][ps], columns permuted by v_col
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

ag_status launch_probe(uint32_t* ids_out, int n_wg, int spin_cycles, hipStream_t st);

// Tokens of context handled by one decode workgroup (one split).
#ifndef AG_DECODE_SPLIT
#define AG_DECODE_SPLIT 512
#endif
constexpr int kDecodeSplit = AG_DECODE_SPLIT;

}  // namespace ag
