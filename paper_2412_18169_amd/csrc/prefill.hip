// Chunked prefill (placeholder until the MFMA kernel lands): entry points reject every call.
#include "kun_internal.h"

extern "C" size_t kun_prefill_workspace_bytes(const kun_kv_pool* p, int n_chunks, int Hq, int total_new_tokens) {
    (void)p; (void)n_chunks; (void)Hq; (void)total_new_tokens;
    return 256;
}

extern "C" int kun_paged_prefill_chunk(kun_kv_pool* p, const void* q, void* out, const int32_t* q_start,
                                       const int32_t* prior_len, const int32_t* block_table, int max_blocks,
                                       int n_chunks, int Hq, int total_new_tokens, float scale,
                                       void* workspace, size_t workspace_bytes, void* stream) {
    return KUN_ERR_UNSUPPORTED;
}
