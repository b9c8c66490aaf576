// KV append: scatter the K/V rows of new tokens into their page slots through the block table.
// K rows are contiguous in a page; V is stored transposed ([dim][token]), so a token's V row
// becomes head_dim strided element stores.  Pure copy: results are bit-exact.
#include "kun_internal.h"

namespace {

template <typename E>
__global__ __launch_bounds__(256) void kv_append_kernel(const KunRanges rt, const E* __restrict__ k_new,
                                                        const E* __restrict__ v_new,
                                                        const int32_t* __restrict__ seq_of_tok,
                                                        const int32_t* __restrict__ pos_of_tok,
                                                        const int32_t* __restrict__ table, int max_blocks,
                                                        int T, int Hkv, int D, int B,
                                                        unsigned block_bytes, unsigned page_bytes) {
    for (int i = blockIdx.x; i < T; i += gridDim.x) {
        const int seq = seq_of_tok[i], pos = pos_of_tok[i];
        const int blk = table[(size_t)seq * max_blocks + pos / B];
        const int slot = pos % B;
        char* block = kun_block_addr(rt, blk, block_bytes);
        for (int x = threadIdx.x; x < Hkv * D; x += blockDim.x) {
            const int h = x / D, j = x - h * D;
            E* page = (E*)(block + (size_t)h * page_bytes);
            page[slot * D + j] = k_new[(size_t)i * Hkv * D + x];
            page[B * D + j * B + slot] = v_new[(size_t)i * Hkv * D + x];
        }
    }
}

}  // namespace

extern "C" int kun_kv_append(kun_kv_pool* p, const void* k_new, const void* v_new,
                             const int32_t* seq_of_tok, const int32_t* pos_of_tok, int T,
                             const int32_t* block_table, int max_blocks, void* stream) {
    if (!p || T < 0) return KUN_ERR_INVALID_ARG;
    if (T == 0) return KUN_OK;
    if (!k_new || !v_new || !seq_of_tok || !pos_of_tok || !block_table || max_blocks <= 0)
        return KUN_ERR_INVALID_ARG;
    const dim3 grid((unsigned)(T < 65536 ? T : 65536));
    hipStream_t st = (hipStream_t)stream;
    if (p->elt == 2)
        hipLaunchKernelGGL(kv_append_kernel<uint16_t>, grid, dim3(256), 0, st, p->ranges,
                           (const uint16_t*)k_new, (const uint16_t*)v_new, seq_of_tok, pos_of_tok,
                           block_table, max_blocks, T, p->Hkv, p->d, p->B, (unsigned)p->block_bytes,
                           (unsigned)p->page_bytes);
    else
        hipLaunchKernelGGL(kv_append_kernel<uint32_t>, grid, dim3(256), 0, st, p->ranges,
                           (const uint32_t*)k_new, (const uint32_t*)v_new, seq_of_tok, pos_of_tok,
                           block_table, max_blocks, T, p->Hkv, p->d, p->B, (unsigned)p->block_bytes,
                           (unsigned)p->page_bytes);
    KUN_HIP_CHECK_LAUNCH();
    return KUN_OK;
}
