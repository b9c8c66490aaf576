// KV append: scatter the K/V rows of new tokens into their page slots through the block table.
// A page is a row of tiles of 16 tokens; K rows are contiguous in a tile, V is stored transposed
// ([dim][token]) behind them, so a token's V row becomes head_dim strided element stores.  Pure copy:
// results are bit-exact.
#include "kun_internal.h"

namespace {

constexpr int kTile = 16;       // tokens per tile of a page

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
        const int tile = (pos % B) / kTile, slot = pos % kTile;
        char* block = kun_block_addr(rt, blk, block_bytes);
        for (int x = threadIdx.x; x < Hkv * D; x += blockDim.x) {
            const int h = x / D, j = x - h * D;
            E* t = (E*)(block + (size_t)h * page_bytes) + (size_t)tile * (2 * kTile * D);
            t[slot * D + j] = k_new[(size_t)i * Hkv * D + x];
            t[kTile * D + j * kTile + slot] = v_new[(size_t)i * Hkv * D + x];
        }
    }
}

// Block resolution as data: where token (seq, pos) of KV head h lives.
__global__ __launch_bounds__(256) void slot_map_kernel(const KunRanges rt, const int32_t* __restrict__ seq_of_tok,
                                                       const int32_t* __restrict__ pos_of_tok,
                                                       const int32_t* __restrict__ table, int max_blocks, int T,
                                                       int h, int D, int B, unsigned elt, unsigned block_bytes,
                                                       unsigned page_bytes, int32_t* __restrict__ range_out,
                                                       int64_t* __restrict__ k_off, int64_t* __restrict__ v_off) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < T; i += gridDim.x * blockDim.x) {
        const int seq = seq_of_tok[i], pos = pos_of_tok[i];
        const int blk = table[(size_t)seq * max_blocks + pos / B];
        const int tile = (pos % B) / kTile, slot = pos % kTile;
        const char* page = kun_block_addr(rt, blk, block_bytes) + (size_t)h * page_bytes +
                           (size_t)tile * (2 * kTile * D) * elt;
        int r = 0;
        for (int j = 1; j < rt.n; ++j)
            if (blk >= rt.first[j]) r = j;
        range_out[i] = r;
        k_off[i] = (int64_t)(page + (size_t)slot * D * elt - rt.base[r]);
        v_off[i] = (int64_t)(page + ((size_t)kTile * D + slot) * elt - rt.base[r]);
    }
}

}  // namespace

extern "C" int kun_slot_map(const kun_kv_pool* p, const int32_t* seq_of_tok, const int32_t* pos_of_tok, int T,
                            const int32_t* block_table, int max_blocks, int kv_head, int32_t* range_out,
                            int64_t* k_off_out, int64_t* v_off_out, void* stream) {
    if (!p || T < 0 || kv_head < 0 || kv_head >= p->Hkv) return KUN_ERR_INVALID_ARG;
    if (T == 0) return KUN_OK;
    if (!seq_of_tok || !pos_of_tok || !block_table || max_blocks <= 0 || !range_out || !k_off_out || !v_off_out)
        return KUN_ERR_INVALID_ARG;
    const int nb = (T + 255) / 256;
    hipLaunchKernelGGL(slot_map_kernel, dim3((unsigned)(nb < 4096 ? nb : 4096)), dim3(256), 0, (hipStream_t)stream,
                       p->ranges, seq_of_tok, pos_of_tok, block_table, max_blocks, T, kv_head, p->d, p->B,
                       (unsigned)p->elt, (unsigned)p->block_bytes, (unsigned)p->page_bytes, range_out, k_off_out,
                       v_off_out);
    KUN_HIP_CHECK_LAUNCH();
    return KUN_OK;
}

extern "C" int kun_kv_append(kun_kv_pool* p, const void* k_new, const void* v_new,
                             const int32_t* seq_of_tok, const int32_t* pos_of_tok, int T,
                             const int32_t* block_table, int max_blocks, void* stream) {
    if (!p || T < 0) return KUN_ERR_INVALID_ARG;
    if (T == 0) return KUN_OK;
    if (!k_new || !v_new || !seq_of_tok || !pos_of_tok || !block_table || max_blocks <= 0)
        return KUN_ERR_INVALID_ARG;
    const dim3 grid((unsigned)(T < 65536 ? T : 65536));
    hipStream_t st = (hipStream_t)stream;
    if (p->elt == 1)
        hipLaunchKernelGGL(kv_append_kernel<uint8_t>, grid, dim3(256), 0, st, p->ranges,
                           (const uint8_t*)k_new, (const uint8_t*)v_new, seq_of_tok, pos_of_tok,
                           block_table, max_blocks, T, p->Hkv, p->d, p->B, (unsigned)p->block_bytes,
                           (unsigned)p->page_bytes);
    else if (p->elt == 2)
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
