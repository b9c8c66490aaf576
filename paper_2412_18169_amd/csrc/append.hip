// KV append: scatter the K/V rows of new tokens into their page slots through the block table.
// A page is a row of tiles of 16 tokens; K rows are contiguous in a tile, V is stored transposed
// ([dim][token]) behind them.  Pure copy: results are bit-exact.
#include "kun_internal.h"

namespace {

constexpr int kTile = 16;       // tokens per tile of a page

// Tokens that follow each other in the input AND in a page tile (same request, consecutive positions,
// same 16-token tile) form a run: a prefill chunk is a sequence of runs of 16, one per tile, a decode
// token is a run of 1.  A run is written by one workgroup: K rows as 16-byte copies, V staged in LDS
// and written as whole V^T rows ([dim][16 tokens]: 32 contiguous bytes per dim in bf16) when the run
// fills its tile, element by element otherwise.  (One 2-byte store per element, as a token-by-token
// scatter does, made the memory system write five times the bytes moved.)
//
// Workgroup (b, kv head) owns the runs whose FIRST token has an input index in [16 b, 16 b + 16); such a
// run ends at most 15 tokens later, so the workgroup looks at the 31 tokens from 16 b on.
constexpr int kGroup = 16;                 // run heads per workgroup
constexpr int kWindow = 2 * kGroup - 1;    // tokens a workgroup may have to move

template <typename E, int D>
__global__ __launch_bounds__(256) void kv_append_kernel(const KunRanges rt, const E* __restrict__ k_new,
                                                        const E* __restrict__ v_new,
                                                        const int32_t* __restrict__ seq_of_tok,
                                                        const int32_t* __restrict__ pos_of_tok,
                                                        const int32_t* __restrict__ table, int max_blocks,
                                                        int T, int Hkv, int B,
                                                        unsigned block_bytes, unsigned page_bytes) {
    constexpr int CH = D * sizeof(E) / 16;             // 16-byte chunks per row
    constexpr int VPR = kTile * sizeof(E) / 16;        // 16-byte stores per full V^T row
    constexpr int NP = (kWindow * CH + 255) / 256;     // 16-byte pieces of the window's rows per thread
    __shared__ char* s_tile[kWindow];                  // address of the token's page tile (this kv head), or null
    __shared__ int s_slot[kWindow], s_head[kWindow];   // slot in the tile; input offset of the token's run head, or -1
    __shared__ int s_len[kGroup];                      // length of the run that starts at offset t (0: none starts there)
    __shared__ __attribute__((aligned(16))) E s_v[kWindow][D];
    const int h = blockIdx.x % Hkv, base = (blockIdx.x / Hkv) * kGroup;
    const int tid = threadIdx.x;

    // The rows of the window are requested first: they depend on nothing, and the chain token -> table
    // entry -> page address, which decides where (and whether) they go, runs under their latency.
    uint4 kreg[NP], vreg[NP];
#pragma unroll
    for (int n = 0; n < NP; ++n) {
        const int x = tid + 256 * n, t = x / CH, c = x % CH;
        kreg[n] = vreg[n] = make_uint4(0, 0, 0, 0);
        if (x < kWindow * CH && base + t < T) {
            const size_t src = ((size_t)(base + t) * Hkv + h) * D * sizeof(E) + (size_t)c * 16;
            kreg[n] = *(const uint4*)((const char*)k_new + src);
            vreg[n] = *(const uint4*)((const char*)v_new + src);
        }
    }

    // Wave 0, lane t = token base + t of the window: its tile and slot, and the runs of the window.
    if (tid < 64) {
        const int i = base + tid;
        char* tile = nullptr;
        int slot = 0;
        bool starts = false;
        if (tid < kWindow && i < T) {
            const int seq = seq_of_tok[i], pos = pos_of_tok[i];
            // A token that its table row cannot place -- row or position below zero, position beyond the
            // row's max_blocks * B tokens, a block id outside the pool -- is left out: nothing is written
            // for it.  (The tokens of one run share their table entry, so a run is placed or left out as
            // a whole.)
            const int blk = (seq >= 0 && pos >= 0 && pos < (long long)max_blocks * B)
                                ? table[(size_t)seq * max_blocks + pos / B] : -1;
            if (blk >= 0 && blk < rt.first[rt.n]) {
                tile = kun_block_addr(rt, blk, block_bytes) + (size_t)h * page_bytes +
                       (size_t)((pos % B) / kTile) * (2 * kTile * D) * sizeof(E);
                slot = pos % kTile;
                // a run starts here unless the token before continues into this slot of this tile
                starts = i == 0 || slot == 0 || seq_of_tok[i - 1] != seq || pos_of_tok[i - 1] != pos - 1;
            }
        }
        // A run ends in front of the next run head, the next token that is left out, or the window's end.
        // Runs whose head lies in [0, kGroup) are this workgroup's; tokens in front of the first head
        // belong to the workgroup before, tokens behind a head at kGroup or later to the next one.
        const bool in_window = tid < kWindow && i < T;
        const unsigned long long heads = __builtin_amdgcn_ballot_w64(starts);
        const unsigned long long breaks = __builtin_amdgcn_ballot_w64(in_window && (starts || !tile));
        const int window_end = min(kWindow, T - base);
        if (tid < kWindow) {
            int head = -1;
            if (tile) {
                const unsigned long long upto = breaks & ((2ull << tid) - 1);      // breaks at or before this token
                if (upto) {
                    const int hb = 63 - __builtin_clzll(upto);
                    if (((heads >> hb) & 1) && hb < kGroup) head = hb;
                }
            }
            s_tile[tid] = tile;
            s_slot[tid] = slot;
            s_head[tid] = head;
        }
        if (tid < kGroup) {
            int len = 0;
            if (starts) {
                const unsigned long long after = breaks & ~((2ull << tid) - 1);
                len = (after ? min(__builtin_ctzll(after), window_end) : window_end) - tid;
            }
            s_len[tid] = len;
        }
    }
    __syncthreads();
    // K rows and staging of V rows: 16-byte pieces
#pragma unroll
    for (int n = 0; n < NP; ++n) {
        const int x = tid + 256 * n, t = x / CH, c = x % CH;
        if (x >= kWindow * CH || s_head[t] < 0) continue;
        *(uint4*)(s_tile[t] + (size_t)s_slot[t] * D * sizeof(E) + c * 16) = kreg[n];
        *(uint4*)((char*)&s_v[t][0] + c * 16) = vreg[n];
    }
    __syncthreads();
    // V^T: thread = (run head, dim)
    for (int x = tid; x < kGroup * D; x += 256) {
        const int hd = x / D, j = x % D;
        const int len = s_len[hd];
        if (len == 0) continue;
        E* row = (E*)(s_tile[hd] + (size_t)kTile * D * sizeof(E)) + (size_t)j * kTile;
        if (len == kTile) {                            // the run fills its tile: one whole row
            union { E e[kTile]; uint4 u[VPR]; } r;
#pragma unroll
            for (int t = 0; t < kTile; ++t) r.e[t] = s_v[hd + t][j];
#pragma unroll
            for (int c = 0; c < VPR; ++c) ((uint4*)row)[c] = r.u[c];
        } else {
            // Non-temporal stores: a decode token's V goes element by element into 128 rows of its tile,
            // 32 cache lines per (token, kv head).  Written with ordinary stores those lines stay behind,
            // dirty, in the L2 of whichever XCD ran this workgroup, and the decode call that reads the tile
            // next pays for it (measured: 512 decode tokens made the following 0.44 ms decode call 20 us
            // longer; with these stores nothing is left of that).
            const int slot0 = s_slot[hd];
            for (int t = 0; t < len; ++t) __builtin_nontemporal_store(s_v[hd + t][j], &row[slot0 + t]);
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
        const int blk = (seq >= 0 && pos >= 0 && pos < (long long)max_blocks * B)
                            ? table[(size_t)seq * max_blocks + pos / B] : -1;
        if (blk < 0 || blk >= rt.first[rt.n]) {            // a token the table row cannot place
            range_out[i] = -1;
            k_off[i] = -1;
            v_off[i] = -1;
            continue;
        }
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
    const dim3 grid((unsigned)((size_t)((T + kGroup - 1) / kGroup) * p->Hkv));
    hipStream_t st = (hipStream_t)stream;
#define KUN_APPEND(E, DD)                                                                                          \
    hipLaunchKernelGGL((kv_append_kernel<E, DD>), grid, dim3(256), 0, st, p->ranges, (const E*)k_new,              \
                       (const E*)v_new, seq_of_tok, pos_of_tok, block_table, max_blocks, T, p->Hkv, p->B,          \
                       (unsigned)p->block_bytes, (unsigned)p->page_bytes)
    if (p->elt == 1) { if (p->d == 128) KUN_APPEND(uint8_t, 128); else KUN_APPEND(uint8_t, 64); }
    else if (p->elt == 2) { if (p->d == 128) KUN_APPEND(uint16_t, 128); else KUN_APPEND(uint16_t, 64); }
    else { if (p->d == 128) KUN_APPEND(uint32_t, 128); else KUN_APPEND(uint32_t, 64); }
#undef KUN_APPEND
    KUN_HIP_CHECK_LAUNCH();
    return KUN_OK;
}
