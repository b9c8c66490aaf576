// Internal definitions shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kun.h"

// Range table handed to every kernel BY VALUE, so that a later kun_kv_pool_extend cannot disturb
// a launch already enqueued.  first[r] is the id of the first block of range r;
// first[n] = total number of blocks.  Unused entries hold INT32_MAX / nullptr.
struct KunRanges {
    int32_t n;
    int32_t first[KUN_MAX_RANGES + 1];
    char* base[KUN_MAX_RANGES];
};

struct kun_kv_pool {
    KunRanges ranges;
    size_t range_bytes[KUN_MAX_RANGES];
    int dtype;        // kun_dtype
    int Hkv, d, B;
    size_t elt;       // bytes per element
    size_t block_bytes;
    size_t page_bytes;   // one (block, kv head): K then V^T
};

// Device address of block `blk` (wave-uniform callers get scalar code).
__device__ __forceinline__ char* kun_block_addr(const KunRanges& rt, int blk, size_t block_bytes) {
    int r = 0;
    for (int i = 1; i < rt.n; ++i)
        if (blk >= rt.first[i]) r = i;
    return rt.base[r] + (size_t)(blk - rt.first[r]) * block_bytes;
}

// Attention of T independent query rows by the vector-ALU decode kernel, any supported dtype and
// head_dim: row t has ctx_len[t] tokens (device int32 [T]) behind row row_of_seq[t] of the block
// table (device int32 [T]); q, out: device [T, Hq, head_dim].  One workgroup per (row, kv head)
// walks the whole context.  workspace: device, 256-byte aligned, kun_attend_rows_workspace_bytes(T).
size_t kun_attend_rows_workspace_bytes(int T);
int kun_attend_rows_generic(const kun_kv_pool* p, const void* q, void* out, const int32_t* table, int max_blocks,
                            const int32_t* ctx_len, const int32_t* row_of_seq, int T, int Hq, float scale,
                            void* workspace, hipStream_t st);

// Process-wide tuning options (kun_set_option): read from the environment once, when the library is
// loaded, and changed only by kun_set_option afterwards; launches read this struct, never the
// environment.
struct KunOptions {
    int decode_part = 0;          // tokens per split-K partition (multiple of 32); 0 = chosen from the bound
    int decode_waves = 4;         // waves per workgroup of the MFMA decode kernel: 1, 2 or 4
    bool decode_generic = false;  // run the vector-ALU decode kernel where the MFMA one would
    bool decode_flat_map = false; // item-major workgroup order instead of the XCD-aware one
    int decode_merge = 0;         // 0 = by batch size, 1 = always inside the partial kernel, 2 = always a launch of its own
    int prefill_shape = 0;        // 0 = default kernel; other values select cross-check kernels (prefill.hip)
};
const KunOptions& kun_options();

// Remembers which HIP call failed and how, per host thread, for kun_last_hip_error().
void kun_note_hip_error(const char* call, hipError_t e);

#define KUN_HIP_CHECK_LAUNCH()                               \
    do {                                                     \
        const hipError_t e_ = hipGetLastError();             \
        if (e_ != hipSuccess) {                              \
            kun_note_hip_error("kernel launch", e_);         \
            return KUN_ERR_HIP;                              \
        }                                                    \
    } while (0)
