// Chunked prefill over paged K/V: bf16 or FP8 (E4M3) pages, bf16 queries, head_dim 128, pages of
// 16-token tiles (blocks of 16 to 128 tokens), MFMA 32x32x16 bf16 with fp32 accumulation.
//
// A chunk of c new tokens after p prior tokens attends to keys 0 .. p + r for its row r
// (Section 4.3, Eq. 1: prefix attention p*c plus causal self attention (c*c + c)/2 pairs).  This is
// the compute-bound part of a serving iteration (Section 2.1), so it runs on the matrix cores.
//
// Work item = (chunk, tile of query positions, kv head).  The G query heads that share the kv head
// are stacked into the row dimension (row = position * G + head), so a K/V tile staged in LDS
// serves all of them.  A workgroup has 8 waves; each wave owns 32 rows and walks the keys in tiles
// of 64 (four page tiles), flash-attention style:
//
//   S^T[key][row]  = K[key][:] . Q[row][:]          A = K fragment from LDS, B = Q in registers
//   online softmax over keys, per row: each lane column holds one row, so max/sum are in-lane
//                                                    plus one exchange between the two lane halves
//   O^T[dim][row] += V^T[dim][key] P^T[key][row]    A = V^T fragment from LDS (pages store V as
//                                                    [dim][token]), B = P straight from the S^T
//                                                    accumulator registers, rounded to bf16
//
// S^T tile rows are mapped to keys so that the 8 accumulator values a lane feeds to one PV MFMA
// are 8 consecutive keys of one page tile, i.e. one 16-byte LDS read of V^T.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "kun_internal.h"

namespace {

constexpr int kBlock = 16;
constexpr int D = 128;
constexpr int BN = 64;                  // keys per LDS tile (4 KV blocks)
constexpr int kBlocksPerTile = BN / kBlock;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.0f;           // log2 of the largest softmax numerator kept without rescaling
constexpr float kSumCap = 8192.0f;      // 32 * 2^kLazy: a lane's 32 numerators can only sum above it if one exceeds 2^kLazy

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

union Frag {
    uint4 u;
    bf16x8 v;
};

struct PrefillArgs {
    KunRanges rt;
    const void* q;
    void* out;
    const int32_t* q_start;
    const int32_t* prior;
    const int32_t* table;
    int32_t* n_items;     // workspace
    int32_t* next_item;   // workspace: 8 counters (one per XCD) for the workgroups that fetch their work
    int2* items;          // workspace: (chunk, position tile)
    // Launches with too few items to fill the chip split the keys of an item over several workgroups:
    const int2* split_info;   // workspace, NULL when the launch cannot need it: per item (split | nsplit << 16, slot)
    const int4* desc;         // workspace: two int4 per list entry, (chunk, position tile, prior tokens, first query row)
                              // and (chunk tokens, first key tile, key tiles, partial-result slot or -1), for the ring kernels
    const unsigned long long* page_addr;   // workspace: [chunk][16-token tile of the request] device address of the tile of
                                           // KV head 0 (block resolution done once per tile, by the plan launch)
    int tiles_per_row;        // entries per chunk in page_addr (page_row_entries)
    int4* split_items;        // workspace: (chunk, position tile, nsplit, first slot) of every split item
    int32_t* n_split_items;   // workspace
    float* part_o;            // workspace: [slot, kvh, 256 rows, 128] unnormalised outputs of a key range
    float* part_ml;           // workspace: [slot, kvh, 256 rows, 2]  (m in log2 units, l)
    int max_blocks;
    int n_chunks, Hkv, Hq;
    int max_items;
    float scale_log2;
    unsigned block_bytes, page_bytes;
    int sub_shift;           // log2 of the 16-token page tiles per KV block (0 .. 3): page tile i of a request is tile i % 2^shift of block i >> shift
    int plan_tag;            // what the plan launch left behind n_items: a call on a workspace without a plan of this
                             // batch shape (kun_paged_prefill_chunk_planned without its plan) computes nothing
};

// sixteen FP8 (E4M3) codes -> two MFMA operands of eight bf16 each (codes 0..7, codes 8..15); exact
__device__ __forceinline__ void fp8x16_to_bf16(const uint4& x, Frag& lo, Frag& hi) {
    union { bf16x2 h; unsigned u; } c[8];
    c[0].h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x.x, 1.0f, false);
    c[1].h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x.x, 1.0f, true);
    c[2].h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x.y, 1.0f, false);
    c[3].h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x.y, 1.0f, true);
    c[4].h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x.z, 1.0f, false);
    c[5].h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x.z, 1.0f, true);
    c[6].h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x.w, 1.0f, false);
    c[7].h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x.w, 1.0f, true);
    lo.u = make_uint4(c[0].u, c[1].u, c[2].u, c[3].u);
    hi.u = make_uint4(c[4].u, c[5].u, c[6].u, c[7].u);
}

// max of three floats in one instruction.  Plain fmaxf makes the compiler canonicalise every MFMA
// output first (one extra v_max per value); the instruction itself already handles NaN inputs.
// The compiler does not add the wait states an MFMA result needs before a vector ALU reads it when
// the reader is inline asm, so `a` must come out of an instruction the compiler generated itself
// after the MFMAs that wrote `b` and `c` (a chain that starts from a plain fmaxf over both
// accumulators): by then every lane of those results has landed.
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
    return (unsigned)f32_to_bf16_rne(a) | ((unsigned)f32_to_bf16_rne(b) << 16);
}

// One workgroup lists the (chunk, position tile) items and orders them by decreasing number of key
// tiles (longest first), so that the ragged causal costs pack well onto the CUs.
constexpr int kPlanThreads = 1024;
constexpr int kPlanSortMax = 4096;      // items beyond this stay in chunk order
constexpr int kPlanBuckets = 1024;      // cost buckets (key tiles); longer ones share the first bucket
constexpr int kSplitTarget = 256;       // split keys when a launch has fewer (item, kv head) workgroups than this
constexpr int kMaxSplit = 16;           // key ranges per item at most
constexpr int kMinTilesPerSplit = 8;    // ... of at least this many 64-key tiles each
constexpr int kSplitRows = 256;         // rows of a workgroup of the kernels that can split (8 waves x 32)

// Block resolution for the whole launch, once per 16-token tile instead of once per (tile, query tile,
// kv head).  A chunk's row has four entries per 64-key tile, for every key tile that its table row can
// hold and one more; the entry of page tile s of key tile kt sits at 4 kt + kun_tile_place(s), so that the
// two page tiles a wave loads (s and s + 2) lie side by side and come with one 16-byte scalar load.
// Entry = address (KV head 0) of 16-token tile min(4 kt + s, last tile of the context) of the request:
// tile t is tile t % (B / 16) of block table[i][t / (B / 16)].  Tiles past the context repeat the last
// one, so the kernels index without a clamp (and every lane issues the same number of loads per tile).
__device__ __host__ constexpr int kun_tile_place(int s) { return s == 1 ? 2 : s == 2 ? 1 : s; }   // its own inverse
__device__ __host__ inline int page_row_entries(int max_blocks, int sub_shift) {
    return (((max_blocks << sub_shift) + kBlocksPerTile - 1) / kBlocksPerTile + 1) * kBlocksPerTile;
}
// New tokens of chunk ch, or 0 if its lengths do not fit together: rows outside [0, total_new), a negative
// prior length, or a context that the chunk's block-table row cannot hold.  Such a chunk is left out
// like an empty one (no kernel then reads a table entry, a query row or a page on its behalf).
__device__ __forceinline__ int chunk_tokens(const int32_t* __restrict__ q_start, const int32_t* __restrict__ prior,
                                            int ch, int total_new, long long row_tokens) {
    const int qs = q_start[ch], qe = q_start[ch + 1], p = prior[ch];
    const bool ok = qs >= 0 && qe > qs && qe <= total_new && p >= 0 && (long long)p + (qe - qs) <= row_tokens;
    return ok ? qe - qs : 0;
}

__device__ void resolve_tiles(const KunRanges& rt, const int32_t* __restrict__ q_start,
                              const int32_t* __restrict__ prior, const int32_t* __restrict__ table, int n_chunks,
                              int max_blocks, int sub_shift, unsigned block_bytes, unsigned tile_bytes,
                              unsigned long long* __restrict__ page_addr, int first_wg, int n_wgs, int total_new,
                              int last_block) {
    const int tiles_per_row = page_row_entries(max_blocks, sub_shift);
    const long long total = (long long)n_chunks * tiles_per_row;
    for (long long e = (long long)(blockIdx.x - first_wg) * blockDim.x + threadIdx.x; e < total;
         e += (long long)n_wgs * blockDim.x) {
        const int ch = (int)(e / tiles_per_row), place = (int)(e % tiles_per_row);
        const int c = chunk_tokens(q_start, prior, ch, total_new, ((long long)max_blocks * kBlock) << sub_shift);
        if (c == 0) continue;
        const int ctx = prior[ch] + c;
        const int last = (ctx - 1) / kBlock;
        int t = (place & ~(kBlocksPerTile - 1)) + kun_tile_place(place & (kBlocksPerTile - 1));
        t = t < last ? t : last;
        // (clamped into the pool: a bad table entry reads some block of the pool, never anything else)
        const int id = min(max(table[(size_t)ch * max_blocks + (t >> sub_shift)], 0), last_block);
        page_addr[e] = (unsigned long long)kun_block_addr(rt, id, block_bytes) +
                       (unsigned)(t & ((1 << sub_shift) - 1)) * tile_bytes;
    }
}

struct ResolveArgs {
    KunRanges rt;
    const int32_t* table;
    unsigned long long* page_addr;
    int max_blocks, sub_shift, n_wgs;
    int total_new;                        // query rows of the call: chunks must lie inside
    int last_block;                       // largest block id of the pool
    unsigned block_bytes, tile_bytes;     // tile_bytes: K and V^T of one 16-token page tile (8192 in bf16, 4096 in FP8)
};

__global__ __launch_bounds__(kPlanThreads) void prefill_plan_kernel(const ResolveArgs ra, const int32_t* __restrict__ q_start,
                                                                  const int32_t* __restrict__ prior, int n_chunks,
                                                                  int pos_per_tile, int max_items,
                                                                  int32_t* __restrict__ n_items,
                                                                  int32_t* __restrict__ next_item,
                                                                  int2* __restrict__ items, int Hkv, int split_target,
                                                                  int max_entries,
                                                                  int2* __restrict__ split_info,
                                                                  int4* __restrict__ split_items,
                                                                  int32_t* __restrict__ n_split_items,
                                                                  int4* __restrict__ desc, int tag) {
    if (blockIdx.x == 0 && threadIdx.x == 0) n_items[1] = tag;
    if (blockIdx.x > 0) {      // workgroups 1 .. n_wgs resolve the blocks; workgroup 0 makes the work list
        resolve_tiles(ra.rt, q_start, prior, ra.table, n_chunks, ra.max_blocks, ra.sub_shift, ra.block_bytes,
                      ra.tile_bytes, ra.page_addr, 1, ra.n_wgs, ra.total_new, ra.last_block);
        return;
    }
    // everything a workgroup needs to know about list entry i, so that it starts with one lookup
    auto write_desc = [&](int i, int2 it, int2 si) {
        const int qs = q_start[it.x], c = q_start[it.x + 1] - qs, p = prior[it.x];
        const int n_tiles = (p + min((it.y + 1) * pos_per_tile, c) - 1) / BN + 1;
        const int split = si.x & 0xffff, nsplit = si.x >> 16;
        const int kt0 = split * n_tiles / nsplit;
        desc[2 * i] = make_int4(it.x, it.y, p, qs);
        desc[2 * i + 1] = make_int4(c, kt0, (split + 1) * n_tiles / nsplit - kt0, si.y);
    };
    __shared__ int base_s;
    __shared__ int cnt[kPlanThreads / 64];               // per-wave totals of the scan
    __shared__ int cost[kPlanSortMax];
    __shared__ int2 tmp_item[kPlanSortMax];
    __shared__ int hist[kPlanBuckets];
    const int tid = threadIdx.x;
    if (tid == 0) base_s = 0;
    if (tid < 8) next_item[tid] = 0;
    __syncthreads();
    for (int c0 = 0; c0 < n_chunks; c0 += kPlanThreads) {
        const int ch = c0 + tid;
        int nt = 0, c = 0, p = 0;
        if (ch < n_chunks) {
            c = chunk_tokens(q_start, prior, ch, ra.total_new, ((long long)ra.max_blocks * kBlock) << ra.sub_shift);
            p = prior[ch];
            nt = (c + pos_per_tile - 1) / pos_per_tile;
        }
        int incl = nt;                                     // inclusive scan inside the wave, then over the waves
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o);
            if ((tid & 63) >= o) incl += y;
        }
        if ((tid & 63) == 63) cnt[tid >> 6] = incl;
        __syncthreads();
        int first = base_s + incl - nt;
        for (int w = 0; w < (tid >> 6); ++w) first += cnt[w];
        for (int t = 0; t < nt; ++t) {
            const int k = first + t;
            if (k >= max_items) break;
            const int last_key = p + min(c, (t + 1) * pos_per_tile) - 1;
            const int2 it = make_int2(ch, t);
            if (k < kPlanSortMax) { cost[k] = last_key / BN + 1; tmp_item[k] = it; }
            else items[k] = it;
        }
        __syncthreads();
        if (tid == kPlanThreads - 1) base_s = first + nt;
        __syncthreads();
    }
    const int total = base_s < max_items ? base_s : max_items;
    const int ns = total < kPlanSortMax ? total : kPlanSortMax;
    // counting sort by decreasing cost: histogram, exclusive scan by one wave, scatter
    for (int i = tid; i < kPlanBuckets; i += kPlanThreads) hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < ns; i += kPlanThreads) {
        const int bkt = kPlanBuckets - 1 - min(cost[i], kPlanBuckets - 1);
        cost[i] = bkt;
        atomicAdd(&hist[bkt], 1);
    }
    __syncthreads();
    if (tid < 64) {
        int carry = 0;
        for (int b0 = 0; b0 < kPlanBuckets; b0 += 64) {
            const int v = hist[b0 + tid];
            int incl = v;
            for (int o = 1; o < 64; o <<= 1) {
                const int y = __shfl_up(incl, o);
                if (tid >= o) incl += y;
            }
            hist[b0 + tid] = carry + incl - v;
            carry += __shfl(incl, 63);
        }
    }
    __syncthreads();
    for (int i = tid; i < ns; i += kPlanThreads) items[atomicAdd(&hist[cost[i]], 1)] = tmp_item[i];
    if (split_target == 0) {
        if (tid == 0) *n_items = total;
        __syncthreads();
        for (int i = tid; i < total; i += kPlanThreads) write_desc(i, items[i], make_int2(1 << 16, -1));
        return;
    }
    // Too few workgroups for the chip (the host only asks when that is possible): give every item up to
    // `want` key ranges of at least kMinTilesPerSplit tiles each and rewrite the list with one entry per
    // (item, key range).  total * Hkv < split_target here, so one thread per item does it.
    __shared__ int nsp_s[kSplitTarget], off_s[kSplitTarget], slot_s[kSplitTarget], idx_s[kSplitTarget];
    __shared__ int n_out_s, n_split_s;
    __syncthreads();
    const int wgs = total * Hkv;
    int want = (wgs > 0 && wgs < split_target) ? (split_target + wgs - 1) / wgs : 1;
    if (want > kMaxSplit) want = kMaxSplit;
    const bool mine = want > 1 && tid < total;             // total < kSplitTarget <= kPlanThreads
    int2 it = make_int2(0, 0);
    if (mine) {
        it = items[tid];                                   // sorted order, written by this workgroup
        const int c = q_start[it.x + 1] - q_start[it.x];
        const int tiles = (prior[it.x] + min(c, (it.y + 1) * pos_per_tile) - 1) / BN + 1;
        nsp_s[tid] = max(1, min(want, tiles / kMinTilesPerSplit));
    }
    __syncthreads();
    if (tid == 0) {
        int n_out = 0, n_split = 0, slot = 0;
        if (want > 1) {
            for (int i = 0; i < total; ++i) {
                off_s[i] = n_out;
                slot_s[i] = slot;
                idx_s[i] = n_split;
                n_out += nsp_s[i];
                if (nsp_s[i] > 1) {
                    slot += nsp_s[i];
                    ++n_split;
                }
            }
            // never beyond what the host sized (cannot happen with its bounds): then nothing is split
            if (n_out > max_entries || slot * Hkv > 2 * split_target + Hkv) want = 1;
        }
        n_out_s = want > 1 ? n_out : total;
        n_split_s = want > 1 ? n_split : 0;
    }
    __syncthreads();
    if (n_split_s == 0 && n_out_s == total) {              // nothing split: every item is its own whole key range
        for (int i = tid; i < total; i += kPlanThreads) split_info[i] = make_int2(1 << 16, -1);
    } else if (mine) {
        const int nsp = nsp_s[tid];
        if (nsp > 1) split_items[idx_s[tid]] = make_int4(it.x, it.y, nsp, slot_s[tid]);
        for (int sp = 0; sp < nsp; ++sp) {
            items[off_s[tid] + sp] = it;
            split_info[off_s[tid] + sp] = make_int2(sp | (nsp << 16), nsp > 1 ? slot_s[tid] + sp : -1);
        }
    }
    if (tid == 0) {
        *n_items = n_out_s;
        *n_split_items = n_split_s;
    }
    __syncthreads();
    for (int i = tid; i < n_out_s; i += kPlanThreads) write_desc(i, items[i], split_info[i]);
}

// ---------------------------------------------------------------------------------------------
// Ring variant (the cross-check of the ping-pong kernel further down, which is the default): 8 waves
// x 32 rows, 64-key tiles in a 4-stage LDS ring filled by direct global->LDS loads (no registers, no
// LDS stores), three tiles in flight, ONE barrier per tile.
//
// Every q tile of a (chunk, kv head) walks the same keys at about the same time, so a tile load sees
// close to the full memory latency, not an L2 hit; the ring keeps ~96 KiB in flight per CU to cover it.
//
//   iteration kt:  wait until this thread's loads of tile kt have landed (two younger tiles stay in
//                  flight)  ->  barrier (all parts of tile kt visible; everybody has left tile kt-1)
//                  ->  issue tile kt+3 into the stage tile kt-1 used  ->  compute tile kt
//
// A lane's 16 bytes land at (wave-uniform LDS base in M0) + 16 * lane, so the K swizzle and the V^T swizzle
// are applied on the global address side.  Loads past the context read the last valid block instead
// (same count of loads per tile for every thread, so the wait counts stay exact); scores of such keys
// are masked and their V^T fragments zeroed before the MFMA.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((address_space(1))) const void* kun_gptr;
typedef __attribute__((address_space(3))) void* kun_lptr;
typedef const __attribute__((address_space(4))) unsigned long long* kun_caddr;   // constant address space: scalar loads

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt = bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
#define KUN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

template <int G, bool PERSIST>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void prefill_ring_kernel(const PrefillArgs a) {
    constexpr int NW = 8, LOADS = 2;                   // 8 waves; page tiles per wave and tile: 2 loads per lane each (K, V^T)
    // Row r of the workgroup is (position r / G, head r % G).  The workgroup holds POS whole positions;
    // when G does not divide its row count the last rows (1 of 256 for G = 3, 5; 4 for G = 6, 7) are
    // dead, and a wave's 32 rows may begin and end in the middle of a position.
    constexpr int ROWS_W = 32, ROWS = NW * ROWS_W, POS = ROWS / G, LIVE = POS * G;
    constexpr int NSTAGE = 4, AHEAD = NSTAGE - 1;
    static_assert(G >= 1 && G <= 16, "1 to 8 or 16 query heads per KV head");

    __shared__ __attribute__((aligned(16))) unsigned char ring[NSTAGE][2 * kBlocksPerTile * 4096];
    constexpr int V_OFF = kBlocksPerTile * 4096;       // V^T pages follow the K pages inside a stage

    // Work index wi = item * Hkv + kvh.  Plain launch: one workgroup per index.  PERSIST: a fixed
    // number of workgroups (a multiple of 8) fetch indices of their own residue class mod 8 -- the XCD
    // the plain launch would have put them on, so K/V of a (chunk, kv head) stays in one L2 -- in
    // increasing order (longest items first) until the list is exhausted; every workgroup then exits.
    __shared__ int s_next;
    int wi = blockIdx.x;
    for (;;) {
    if (PERSIST) {
        __syncthreads();                               // everybody has left the previous item's ring
        if (threadIdx.x == 0) s_next = atomicAdd(&a.next_item[blockIdx.x & 7], 1) * 8 + (blockIdx.x & 7);
        __syncthreads();
        wi = s_next;
    }
    const int item = wi / a.Hkv, kvh = wi % a.Hkv;
    const int2 hdr = *(const int2*)a.n_items;          // list length, tag of the plan that wrote it
    if (hdr.y != a.plan_tag) return;
    if (PERSIST && item >= hdr.x) return;              // (fetched indices can run past the list's capacity)
    const int n_items = PERSIST ? item + 1 : hdr.x;        // plain launch: the grid is within the capacity, so the
    const int4 d0 = a.desc[2 * item], d1 = a.desc[2 * item + 1];     // entry is read together with the list's length
    if (item >= n_items) return;
    const int chunk = d0.x, qt = d0.y, p = d0.z, qs = d0.w, c = d1.x;
    const int kt0 = d1.y, nt = d1.z, part_slot = d1.w;   // this workgroup's key tiles: all of the item's, or one of its key ranges
    const int ctx = p + c;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, jh = lane >> 5;
    const int pos0 = qt * POS;
    const int wpos0 = pos0 + wave * ROWS_W / G;                                  // first position the wave touches
    const int wpos_end = pos0 + min((wave * ROWS_W + ROWS_W - 1) / G, POS - 1) + 1;  // one past its last live one

    // Addresses of the 16-token page tiles of this chunk's request, resolved by the plan launch; read
    // with scalar loads (wave-uniform index), one tile ahead of the loads that use them.
    const kun_caddr arow = (kun_caddr)(a.page_addr + (size_t)chunk * a.tiles_per_row);
    const int ntile_ctx = (ctx + kBlock - 1) / kBlock;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);

    // per-lane source offsets inside a block for the slot this lane fills (slot = (wave % 4) * 64 + lane),
    // the kv head's page included
    const int slot = (wave & 3) * 64 + lane;
    const unsigned k_src = kvh * a.page_bytes + (slot >> 4) * 256 + (((slot & 15) ^ (slot >> 4)) * 16);
    const unsigned v_src = kvh * a.page_bytes + 4096 + ((slot ^ ((slot >> 4) & 1)) * 16);

    // The loads are issued through inline asm: the compiler then neither tracks them nor adds waits of
    // its own in front of LDS reads; completion is tracked by hand with vmcnt (see the tile loop).
    // Address = 64-bit scalar tile address + 32-bit lane offset; LDS destination = M0 + 16 * lane.
    auto dma16 = [&](unsigned long long page, unsigned off, unsigned lds_addr) {
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(page), "s"(lds_addr)
                     : "memory", "m0");
    };
    const unsigned ring_addr = (unsigned)(size_t)(kun_lptr)&ring[0][0];
    // A tile is 4 loads per lane: this wave brings quarter (wave % 4) of K and of V^T of the tile's page
    // tiles wave / 4 and wave / 4 + 2.  Tiles past the context re-read the last one (every lane issues the
    // same number of loads per tile, so the wait counts stay exact).
    auto tile_addr = [&](int j, int i) -> unsigned long long {     // j: tile index relative to kt0
        return arow[(kt0 + j) * kBlocksPerTile + kun_tile_place((wave_u >> 2) + 2 * i)];
    };
    unsigned long long pg0 = tile_addr(0, 0), pg1 = tile_addr(0, 1);      // of the tile to be issued next
    auto issue = [&](int j) {
        const unsigned st = ring_addr + (j % NSTAGE) * (2 * kBlocksPerTile * 4096) + (wave_u & 3) * 1024;
        const unsigned d0 = st + (wave_u >> 2) * 4096, d1 = d0 + 2 * 4096;
        dma16(pg0, k_src, d0);
        dma16(pg0, v_src, d0 + V_OFF);
        dma16(pg1, k_src, d1);
        dma16(pg1, v_src, d1 + V_OFF);
        pg0 = tile_addr(j + 1, 0);
        pg1 = tile_addr(j + 1, 1);
    };

    // ---- prologue: the first AHEAD tiles go in flight, then Q ------------------------------------
    issue(0);
    if (nt > 1) issue(1);
    if (nt > 2) issue(2);

    Frag qf[8];
    int pos = pos0 + (wave * ROWS_W + n) / G;
    const int g_head = (wave * ROWS_W + n) % G;
    const bool live_row = wave * ROWS_W + n < LIVE && pos < c;
    if (!live_row) pos = min(wpos0, c - 1);            // a dead row repeats a row the wave (or the chunk) does have
    const int vis = p + pos;                           // last key this lane's row sees
    {
        const char* qrow = (const char*)a.q + (((size_t)(qs + pos)) * a.Hq + kvh * G + g_head) * (D * 2);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks].u = *(const uint4*)(qrow + (2 * ks + jh) * 16);
    }
    const int wave_vis_max = p + min(wpos_end, c) - 1;
    const int wave_vis_min = p + min(wpos0, c - 1);

    f32x16 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
    float m = -INFINITY, l = 0.f;                      // m in log2 units

    const int krow = 16 * (n >> 4) + 8 * ((n >> 2) & 1) + 4 * ((n >> 3) & 1) + (n & 3);
    const int krow_blk = krow >> 4, krow_in = krow & 15;
    const unsigned k_lane = krow_blk * 4096 + krow_in * 256;
    const unsigned v_lane = V_OFF + n * 32 + ((jh ^ ((n >> 3) & 1)) * 16);
    const float sl2 = a.scale_log2;

    // all of this wave's work on the 64-key tile kt, which sits in `stage_base`
    auto compute = [&](int kt, const unsigned char* stage_base) {
        if (kt > kt0 && kt * BN + BN - 1 <= wave_vis_min) {
            // Fast path, the whole 64-key tile is visible to every row of the wave (no mask, no dead
            // keys) and the rows have a reference maximum m from an earlier tile of this key range.  Both sub-tiles go
            // through each phase together: 16 QK^T MFMAs in two independent chains, one softmax pass
            // over 32 values per lane, 16 PV MFMAs.  No maximum is taken: the row sums, needed anyway,
            // show when a row's scores have outgrown its reference (sum of 32 numerators above
            // 32 * 2^kLazy, or not a number after an overflow of exp2), and only
            // then are the tile's scores taken again with a new reference.  All 16 K fragments are requested before
            // the first MFMA and all 16 V^T fragments before the softmax, so one LDS latency is paid
            // per phase instead of one per pair of MFMAs.
            f32x16 sa, sb;
            const unsigned char* kbase = stage_base + k_lane;
            Frag ka[8], kb[8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const unsigned off = ((2 * ks + jh) ^ krow_in) * 16;
                ka[ks].u = *(const uint4*)(kbase + off);
                kb[ks].u = *(const uint4*)(kbase + 8192 + off);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i) { sa[i] = 0.f; sb[i] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks].v, qf[ks].v, sa, 0, 0, 0);
                sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[ks].v, qf[ks].v, sb, 0, 0, 0);
            }
            const unsigned char* vbase = stage_base + v_lane;
            Frag vf[16];                               // requested in two halves to stay inside the register file
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) vf[4 * h + dt].u = *(const uint4*)(vbase + h * 4096 + dt * 1024);
            __builtin_amdgcn_sched_barrier(0);
            float ps0 = 0.f, ps1 = 0.f, ps2 = 0.f, ps3 = 0.f;
            union { bf16x2 h[16]; uint4 u[4]; } cv;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(sa[i], sl2, -m)), p1 = __builtin_amdgcn_exp2f(fmaf(sa[i + 1], sl2, -m));
                const float p2 = __builtin_amdgcn_exp2f(fmaf(sb[i], sl2, -m)), p3 = __builtin_amdgcn_exp2f(fmaf(sb[i + 1], sl2, -m));
                ps0 += p0; ps1 += p1; ps2 += p2; ps3 += p3;
                cv.h[i >> 1] = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
                cv.h[8 + (i >> 1)] = __builtin_convertvector((f32x2){p2, p3}, bf16x2);
            }
            float pt = (ps0 + ps1) + (ps2 + ps3);
            if (__builtin_amdgcn_ballot_w64(!(pt <= kSumCap)) != 0) {
                // rare: some row outgrew its reference.  Take the scores again, move the reference of
                // those rows and redo the numerators.
#pragma unroll
                for (int i = 0; i < 16; ++i) { sa[i] = 0.f; sb[i] = 0.f; }
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const unsigned off = ((2 * ks + jh) ^ krow_in) * 16;
                    Frag k0, k1;
                    k0.u = *(const uint4*)(kbase + off);
                    k1.u = *(const uint4*)(kbase + 8192 + off);
                    sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0.v, qf[ks].v, sa, 0, 0, 0);
                    sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1.v, qf[ks].v, sb, 0, 0, 0);
                }
                float mx = fmaxf(sa[0], sb[0]);        // the chain's first read of both accumulators
#pragma unroll
                for (int i = 1; i < 16; ++i) mx = max3(mx, sa[i], sb[i]);
                {
                    auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                    mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                }
                const float mxs = mx * sl2;
                const float mn = (mxs > m + kLazy) ? mxs : m;
                const float alpha = __builtin_amdgcn_exp2f(m - mn);
                l *= alpha;
                m = mn;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) o[dt] *= alpha;
                ps0 = ps1 = ps2 = ps3 = 0.f;
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(sa[i], sl2, -m)), p1 = __builtin_amdgcn_exp2f(fmaf(sa[i + 1], sl2, -m));
                    const float p2 = __builtin_amdgcn_exp2f(fmaf(sb[i], sl2, -m)), p3 = __builtin_amdgcn_exp2f(fmaf(sb[i + 1], sl2, -m));
                    ps0 += p0; ps1 += p1; ps2 += p2; ps3 += p3;
                    cv.h[i >> 1] = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
                    cv.h[8 + (i >> 1)] = __builtin_convertvector((f32x2){p2, p3}, bf16x2);
                }
                pt = (ps0 + ps1) + (ps2 + ps3);
            }
            l += pt;
#pragma unroll
            for (int h = 2; h < 4; ++h)
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) vf[4 * h + dt].u = *(const uint4*)(vbase + h * 4096 + dt * 1024);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int h = 0; h < 4; ++h) {              // the four KV blocks of the tile
                Frag pb;
                pb.u = cv.u[h];
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[4 * h + dt].v, pb.v, o[dt], 0, 0, 0);
            }
            return;
        }
#pragma unroll
        for (int st = 0; st < BN / 32; ++st) {
            const int key0 = kt * BN + st * 32;
            if (key0 > wave_vis_max) continue;
            f32x16 s;
#pragma unroll
            for (int i = 0; i < 16; ++i) s[i] = 0.f;
            const unsigned char* kbase = stage_base + st * 8192 + k_lane;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                Frag kf;
                kf.u = *(const uint4*)(kbase + (((2 * ks + jh) ^ krow_in) * 16));
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.v, qf[ks].v, s, 0, 0, 0);
            }
            // register i <-> key key0 + 16 (i/8) + 8 jh + i%8
            if (key0 + 31 > wave_vis_min) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = key0 + 16 * (i >> 3) + 8 * jh + (i & 7);
                    if (key > vis) s[i] = -INFINITY;
                }
            }
            float mx = fmaxf(s[0], s[1]);              // the chain's first read of the accumulator
#pragma unroll
            for (int i = 2; i < 16; i += 2) mx = max3(mx, s[i], s[i + 1]);
            {
                auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            }
            const float mxs = mx * sl2;
            const bool grow = mxs > m + kLazy;         // also true on the first sub-tile (m = -inf)
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float mn = grow ? mxs : m;
                const float alpha = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mn);   // o and l are 0 then
                l *= alpha;
                m = mn;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) o[dt] *= alpha;
            }
            float ps0 = 0.f, ps1 = 0.f;
            union { bf16x2 h[8]; uint4 u[2]; } cv;
            // a row that has seen no key yet (only possible in a key range that does not start at key 0)
            // still has m = -inf and only -inf scores: keep -inf - (-inf) out of the exponent
            const float mref = (m == -INFINITY) ? 0.f : m;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s[i], sl2, -mref));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s[i + 1], sl2, -mref));
                ps0 += p0;
                ps1 += p1;
                cv.h[i >> 1] = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
            }
            l += ps0 + ps1;
            Frag pb[2];
            pb[0].u = cv.u[0];
            pb[1].u = cv.u[1];
            const bool tail = key0 + 32 > ctx;         // keys past the context: their V^T may hold anything
            const unsigned char* vbase = stage_base + st * 8192 + v_lane;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    Frag vf;
                    vf.u = *(const uint4*)(vbase + h * 4096 + dt * 1024);
                    if (tail) {                        // 0 * NaN = NaN: zero the fragment's dead keys
                        const int t0 = key0 + 16 * h + 8 * jh;
                        unsigned x[4] = {vf.u.x, vf.u.y, vf.u.z, vf.u.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (t0 + e >= ctx) x[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                        vf.u = make_uint4(x[0], x[1], x[2], x[3]);
                    }
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pb[h].v, o[dt], 0, 0, 0);
                }
            }
        }
    };

#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks].v));   // q landed before the loop

    for (int j = 0; j < nt; ++j) {
        // this thread's loads of tile j are older than those of the AHEAD - 1 tiles issued after it
        constexpr int LPT = 2 * LOADS;                 // loads per lane and tile
        if (AHEAD > 2 && j + 2 < nt) KUN_WAIT_VMCNT(2 * LPT);
        else if (AHEAD > 1 && j + 1 < nt) KUN_WAIT_VMCNT(LPT);
        else KUN_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();                  // tile j complete in LDS; everybody has left tile j-1
        if (j + AHEAD < nt) issue(j + AHEAD);                    // into the stage tile j-1 used
        compute(kt0 + j, &ring[j % NSTAGE][0]);
    }

    const float lt = l + __shfl_xor(l, 32);
    if (part_slot >= 0) {
        // one key range of a split item: unnormalised O^T ([dim][row]: a register's 32 lanes are 32
        // consecutive rows) and the rows' (m, l), for prefill_merge_kernel
        const size_t wg_rec = (size_t)part_slot * a.Hkv + kvh;
        float* po = a.part_o + wg_rec * (D * kSplitRows) + wave * ROWS_W + n;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) po[(32 * dt + 8 * (i >> 2) + 4 * jh + (i & 3)) * kSplitRows] = o[dt][i];
        if (jh == 0) *(float2*)(a.part_ml + (wg_rec * kSplitRows + wave * ROWS_W + n) * 2) = make_float2(m, lt);
    }
    const float inv = 1.0f / lt;
    if (live_row && part_slot < 0) {
        char* orow = (char*)a.out + (((size_t)(qs + pos)) * a.Hq + kvh * G + g_head) * (D * 2);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int dim = 32 * dt + 8 * i4 + 4 * jh;
                union { bf16x2 h[2]; uint2 u; } w;
                w.h[0] = __builtin_convertvector((f32x2){o[dt][4 * i4 + 0] * inv, o[dt][4 * i4 + 1] * inv}, bf16x2);
                w.h[1] = __builtin_convertvector((f32x2){o[dt][4 * i4 + 2] * inv, o[dt][4 * i4 + 3] * inv}, bf16x2);
                *(uint2*)(orow + dim * 2) = w.u;
            }
    }
    if (!PERSIST) return;
    }
}


// ---------------------------------------------------------------------------------------------
// Ping-pong variant: the same tiling (8 waves x 32 rows, 64-key tiles, 4-stage LDS ring, direct
// global->LDS loads), but the two waves that share a SIMD (wave w and w + 4) run half a tile apart:
// while one is in its matrix phase M(t) = { O^T += V^T(t-1) P^T(t-1) ; S^T(t) = K(t) Q^T }, 32 MFMAs
// back to back, the other is in its vector phase V(t') = softmax numerators of tile t', page-address
// loads and the tile loads.  Two waves that both follow one barrier per tile stay in lock step and
// leave the matrix pipe idle whenever both are in their softmax; here every phase boundary is an
// s_barrier of the whole workgroup and group 1 (waves 4-7) starts one barrier late:
//
//   barrier      b0      b1      b2      b3      b4            b(2nt)   b(2nt+1)
//   waves 0-3    | M(0)  | V(0)  | M(1)  | V(1)  | M(2) ...    | M(nt)  |
//   waves 4-7    |       | M(0)  | V(0)  | M(1)  | V(1) ...    | V(nt-1)| M(nt)
//
// Ring stage t % 4 holds what M(t) reads: K of tile t and V^T of tile t-1 (loaded together, four loads
// per lane as before), so a stage is busy for one and a half tile times; stage t + 4 is requested right
// after b(2t + 2), when M(t) of both groups is over (waves 4-7 at the start of their V(t), waves 0-3 at
// the start of their M(t + 1)), and has to be complete at b(2t + 7): two and a half tile times.
// Inside M every MFMA is paired with one LDS fragment read that is used four MFMAs later
// (sched_group_barrier); the first four fragments are requested in the vector phase before, so the
// phase runs at the rate of the matrix pipe from its first instruction.
// ---------------------------------------------------------------------------------------------
//
// F8: the pages hold FP8 (E4M3) codes, one byte per element (queries and outputs stay bf16).  Every
// stage is widened to bf16 ONCE, into a ring of three bf16 stages with the layout of the bf16 kernel,
// so the matrix phases are the bf16 kernel's own.  (A matrix phase that widens the fragments it reads
// does the work eight times over, once per wave: 256 conversions per wave and tile against 32 here.)
// The codes land in a small ring of the wave's own (three stages of 2 KiB per wave: the half page tile
// of K and of V^T that the wave requests, two loads per lane and stage), and a lane widens the two
// 16-byte pieces it requested itself: between landing and widening there is nothing to agree on with
// other waves, only the wave's own vmcnt.  The widening sits between the MFMAs of a full matrix phase
// (two LDS reads, sixteen conversions, four LDS writes per lane): waves 0-3 widen stage t + 2 in their
// M(t + 1), waves 4-7 stage t + 3 in theirs, both one barrier before the first read of that stage.
template <int G, bool PERSIST, bool F8>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void prefill_pp_kernel(const PrefillArgs a) {
    constexpr int NW = 8, ROWS_W = 32, ROWS = NW * ROWS_W, POS = ROWS / G, LIVE = POS * G;
    constexpr int TILE_B = 4096;                       // bytes of K (or of V^T) of one 16-token page tile in the ring
    constexpr int NSTAGE = F8 ? 3 : 4, STAGE_BYTES = 2 * kBlocksPerTile * TILE_B, V_OFF = kBlocksPerTile * TILE_B;
    // F8: the ring the codes land in: per stage, wave w owns bytes [2048 w, 2048 w + 2048): 1 KiB of K, 1 KiB of V^T
    constexpr int LAND_STAGE = 8 * 2048, LAND_V = 1024;
    constexpr int LPS = F8 ? 2 : 4;                    // loads per lane and stage
#ifndef KUN_PP_AHEAD
#define KUN_PP_AHEAD 4
#endif
#ifndef KUN_PP_PRE
#define KUN_PP_PRE 4
#endif
    constexpr int kAhead = KUN_PP_AHEAD;               // distance, in MFMAs, between a fragment read and its use
    constexpr int kPre = KUN_PP_PRE;                   // V^T fragments requested before the matrix phase begins
    static_assert(G >= 1 && G <= 16, "1 to 8 or 16 query heads per KV head");

    __shared__ __attribute__((aligned(16))) unsigned char ring[NSTAGE][STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char land[F8 ? NSTAGE : 1][F8 ? LAND_STAGE : 16];
    __shared__ int s_next;
    int wi = blockIdx.x;
    for (;;) {
    if (PERSIST) {
        __syncthreads();                               // everybody has left the previous item's ring
        if (threadIdx.x == 0) s_next = atomicAdd(&a.next_item[blockIdx.x & 7], 1) * 8 + (blockIdx.x & 7);
        __syncthreads();
        wi = s_next;
    }
    wi = __builtin_amdgcn_readfirstlane(wi);
    const int item = wi / a.Hkv, kvh = wi % a.Hkv;
    const int2 hdr = *(const int2*)a.n_items;          // list length, tag of the plan that wrote it
    if (hdr.y != a.plan_tag) return;
    if (PERSIST && item >= hdr.x) return;
    const int n_items = PERSIST ? item + 1 : hdr.x;
    const int4 d0 = a.desc[2 * item], d1 = a.desc[2 * item + 1];
    if (item >= n_items) return;
    const int chunk = d0.x, qt = d0.y, p = d0.z, qs = d0.w, c = d1.x;
    const int kt0 = d1.y, nt = d1.z, part_slot = d1.w;
    const int ctx = p + c;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, jh = lane >> 5;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int group = wave_u >> 2;                     // 0: waves 0-3, 1: waves 4-7 (one barrier behind)
    const int pos0 = qt * POS;
    const int wpos0 = pos0 + wave_u * ROWS_W / G;
    const int wpos_end = pos0 + min((wave_u * ROWS_W + ROWS_W - 1) / G, POS - 1) + 1;

    const kun_caddr arow = (kun_caddr)(a.page_addr + (size_t)chunk * a.tiles_per_row);
    const int slot = (wave & 3) * 64 + lane;
    // bf16: this lane fills 16-byte slot `slot` of a page tile's K and V^T (K chunk XOR row, V^T halves swapped).
    // F8: wave w brings half w % 2 of page tile w / 2, K and V^T as they lie in the page.
    const unsigned k_src = F8 ? kvh * a.page_bytes + (64 * (wave & 1) + lane) * 16
                              : kvh * a.page_bytes + (slot >> 4) * 256 + (((slot & 15) ^ (slot >> 4)) * 16);
    const unsigned v_src = F8 ? kvh * a.page_bytes + 2048 + (64 * (wave & 1) + lane) * 16
                              : kvh * a.page_bytes + 4096 + ((slot ^ ((slot >> 4) & 1)) * 16);
    auto dma16 = [&](unsigned long long page, unsigned off, unsigned lds_addr) {
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(page), "s"(lds_addr)
                     : "memory", "m0");
    };
    const unsigned ring_addr = F8 ? (unsigned)(size_t)(kun_lptr)&land[0][0] : (unsigned)(size_t)(kun_lptr)&ring[0][0];
    // bf16: page tiles wave / 4 and wave / 4 + 2 of key tile j (relative to kt0); F8: page tile wave / 2;
    // clamped into the context
    // (the table repeats the context's last page tile behind it; bf16: both addresses with one scalar load)
    typedef unsigned long long AddrPair __attribute__((ext_vector_type(2)));
    unsigned long long kpg0, kpg1;
    auto tile_addr = [&](int j) {
        if (F8) {
            kpg0 = kpg1 = arow[(kt0 + j) * kBlocksPerTile + kun_tile_place(wave_u >> 1)];
        } else {
            const AddrPair pr = *(const __attribute__((address_space(4))) AddrPair*)(arow + (kt0 + j) * kBlocksPerTile + 2 * (wave_u >> 2));
            kpg0 = pr.x;
            kpg1 = pr.y;
        }
    };
    // Stage t: K of key tile t and V^T of key tile t - 1.  kpg: page tiles of key tile `next_t`, vpg: of
    // key tile next_t - 1 (what the next call of issue() sends).
    tile_addr(0);
    unsigned long long vpg0 = kpg0, vpg1 = kpg1;
    unsigned next_t = 0;                               // next stage to request
    auto issue = [&]() {
        if (F8) {
            const unsigned dst = ring_addr + (next_t % NSTAGE) * LAND_STAGE + wave_u * 2048;
            dma16(kpg0, k_src, dst);
            dma16(vpg0, v_src, dst + LAND_V);
        } else {
            const unsigned st = ring_addr + (next_t & 3) * STAGE_BYTES + (wave_u & 3) * 1024;
            const unsigned dst0 = st + (wave_u >> 2) * 4096, dst1 = dst0 + 2 * 4096;
            dma16(kpg0, k_src, dst0);
            dma16(vpg0, v_src, dst0 + V_OFF);
            dma16(kpg1, k_src, dst1);
            dma16(vpg1, v_src, dst1 + V_OFF);
        }
        vpg0 = kpg0;
        vpg1 = kpg1;
        ++next_t;
        tile_addr((int)next_t);
    };
    // stages 0 .. nt exist; `landed(t)`: this lane's loads of stage t are complete (stages are requested
    // in order, four loads each, so everything but the 4 * (next_t - 1 - t) youngest loads is waited for)
    auto landed = [&](int t) {
        const int younger = (int)next_t - 1 - t;
        if (younger == 2) KUN_WAIT_VMCNT(2 * LPS);     // (the usual case first)
        else if (younger >= 3) KUN_WAIT_VMCNT(3 * LPS);
        else if (younger == 1) KUN_WAIT_VMCNT(LPS);
        else KUN_WAIT_VMCNT(0);
    };

    // ---- prologue ---------------------------------------------------------------------------------
    issue();
    if (nt >= 1) issue();
    if (nt >= 2) issue();
    if (!F8 && nt >= 3) issue();                       // (F8: the landing ring has three stages)

    Frag qf[8];
    int pos = pos0 + (wave * ROWS_W + n) / G;
    const int g_head = (wave * ROWS_W + n) % G;
    const bool live_row = wave * ROWS_W + n < LIVE && pos < c;
    if (!live_row) pos = min(wpos0, c - 1);
    const int vis = p + pos;
    {
        const char* qrow = (const char*)a.q + (((size_t)(qs + pos)) * a.Hq + kvh * G + g_head) * (D * 2);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            qf[ks].u = *(const uint4*)(qrow + (2 * ks + jh) * 16);
    }
    const int wave_vis_min = p + min(wpos0, c - 1);

    f32x16 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
    float m = -INFINITY, l = 0.f;                      // m in log2 units

    // key (inside a 32-key sub-tile) of row n of an S^T tile: accumulator register i of a lane is key
    // 16 (i / 8) + 8 jh + i % 8
    const int krow = 16 * (n >> 4) + 8 * ((n >> 2) & 1) + 4 * ((n >> 3) & 1) + (n & 3);
    const int krow_blk = krow >> 4, krow_in = krow & 15;
    const unsigned k_lane = krow_blk * 4096 + krow_in * 256;
    const unsigned v_lane = V_OFF + n * 32 + ((jh ^ ((n >> 3) & 1)) * 16);
    const float sl2 = a.scale_log2;
    // F8: the two 16-byte pieces of codes this lane requests and widens per stage, and where their halves
    // go in the bf16 stage.  Wave w has half w % 2 of page tile w / 2.  K piece: key row 8 (w % 2) +
    // lane / 8, dims 16 (lane % 8) .. + 16 -> two 16-byte chunks, placed XOR the row like the bf16 loads
    // place them; V^T piece: the sixteen tokens of dim 64 (w % 2) + lane -> the dim's two halves, swapped
    // where the bf16 loads swap them.
    // (the second half of a piece goes to the neighbouring chunk: its offset is the first one's XOR 16)
    unsigned w_src = 0, w_dst_k = 0, w_dst_v = 0;
    if (F8) {
        const int pt = wave >> 1, hf = wave & 1;
        const int row = 8 * hf + (lane >> 3), c = lane & 7, dim = 64 * hf + lane, sw = (dim >> 3) & 1;
        w_src = wave * 2048 + lane * 16;
        w_dst_k = pt * 4096 + row * 256 + (((2 * c) ^ row) * 16);
        w_dst_v = V_OFF + pt * 4096 + (((2 * dim) ^ sw) * 16);
    }

    f32x16 sa, sb;                                     // S^T of the tile between its M and its V phase
    union { bf16x2 h[16]; uint4 u[4]; } cv;            // P^T of the tile between its V and the next M phase

    // ---- matrix phase of stage t: PV of key tile t - 1, QK^T of key tile t --------------------------
    // The first kPre V^T fragments were requested in the vector phase before (prefetch_v), so the first
    // MFMAs find their operands; from then on every MFMA is followed by the read of a fragment that is
    // used kPre MFMAs later.
    Frag vpre[kPre];
    auto prefetch_v = [&](int t) {
        const unsigned char* vbase = &ring[F8 ? t % NSTAGE : t & 3][0] + v_lane;
#pragma unroll
        for (int i = 0; i < kPre; ++i) vpre[i].u = *(const uint4*)(vbase + (i >> 2) * 4096 + (i & 3) * 1024);
    };
    auto mphase = [&](int t, auto do_pv, auto do_qk) {
        const unsigned char* stage = &ring[F8 ? t % NSTAGE : t & 3][0];
        const unsigned char* vbase = stage + v_lane;
        const unsigned char* kbase = stage + k_lane;
        constexpr bool PV = decltype(do_pv)::value, QK = decltype(do_qk)::value;
        constexpr bool W = F8 && PV && QK;             // the full phase also widens this lane's pieces of stage t + 1 + group
        uint4 raw0, raw1;
        if constexpr (W) {
            const unsigned char* src = &land[F8 ? (t + 1 + group) % NSTAGE : 0][0] + w_src;
            raw0 = *(const uint4*)src;
            raw1 = *(const uint4*)(src + LAND_V);
        }
        Frag vf[16], ka[8], kb[8];
        if (PV) {
#pragma unroll
            for (int i = kPre; i < 16; ++i) vf[i].u = *(const uint4*)(vbase + (i >> 2) * 4096 + (i & 3) * 1024);
        }
        if (QK) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const unsigned off = ((2 * ks + jh) ^ krow_in) * 16;
                ka[ks].u = *(const uint4*)(kbase + off);
                kb[ks].u = *(const uint4*)(kbase + 8192 + off);
            }
        }
        if (PV) {
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                Frag pb;
                pb.u = cv.u[h];
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(4 * h + dt < kPre ? vpre[(4 * h + dt) % kPre].v : vf[4 * h + dt].v,
                                                                    pb.v, o[dt], 0, 0, 0);
            }
        }
        if (QK) {
#pragma unroll
            for (int i = 0; i < 16; ++i) { sa[i] = 0.f; sb[i] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks].v, qf[ks].v, sa, 0, 0, 0);
                sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[ks].v, qf[ks].v, sb, 0, 0, 0);
            }
        }
        if constexpr (W) {
            unsigned char* dst = &ring[(t + 1 + group) % NSTAGE][0];
            Frag lo, hi;
            fp8x16_to_bf16(raw0, lo, hi);
            *(uint4*)(dst + w_dst_k) = lo.u;
            *(uint4*)(dst + (w_dst_k ^ 16)) = hi.u;
            fp8x16_to_bf16(raw1, lo, hi);
            *(uint4*)(dst + w_dst_v) = lo.u;
            *(uint4*)(dst + (w_dst_v ^ 16)) = hi.u;
        }
        constexpr int NM = (PV ? 16 : 0) + (QK ? 16 : 0);       // MFMAs
        constexpr int NR = (PV ? 16 - kPre : 0) + (QK ? 16 : 0);   // fragment reads inside the phase
        constexpr int LEAD = PV ? 0 : kAhead;                   // reads in front of the first MFMA
        // (W: the two reads of codes first; the conversions fall between the MFMAs, the four writes of the
        // widened pieces behind MFMAs 12, 16, 20 and 24)
        __builtin_amdgcn_sched_group_barrier(0x100, LEAD + (W ? 2 : 0), 0);
#pragma unroll
        for (int i = 0; i < NR - LEAD; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NM - (NR - LEAD), 0);
    };
    // PV of the context's last key tile when it holds keys past the context (once per item at most)
    auto pv_tail = [&](int t) {
        const unsigned char* vbase = &ring[F8 ? t % NSTAGE : t & 3][0] + v_lane;
        const int key0 = (kt0 + t - 1) * BN;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            Frag pb;
            pb.u = cv.u[h];
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                Frag vf;
                vf.u = *(const uint4*)(vbase + h * 4096 + dt * 1024);
                const int t0 = key0 + 16 * h + 8 * jh;
                unsigned x[4] = {vf.u.x, vf.u.y, vf.u.z, vf.u.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (t0 + e >= ctx) x[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                vf.u = make_uint4(x[0], x[1], x[2], x[3]);
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pb.v, o[dt], 0, 0, 0);
            }
        }
    };

    // ---- vector phase of key tile t: softmax numerators of sa / sb -> cv, row sums, lazy maximum ----
    // Accumulator register i of sa <-> key 64 kt + 16 (i / 8) + 8 jh + i % 8, of sb 32 keys further on.
    auto numerators = [&](float mref) -> float {
        float ps0 = 0.f, ps1 = 0.f, ps2 = 0.f, ps3 = 0.f;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(sa[i], sl2, -mref)), p1 = __builtin_amdgcn_exp2f(fmaf(sa[i + 1], sl2, -mref));
            const float p2 = __builtin_amdgcn_exp2f(fmaf(sb[i], sl2, -mref)), p3 = __builtin_amdgcn_exp2f(fmaf(sb[i + 1], sl2, -mref));
            ps0 += p0; ps1 += p1; ps2 += p2; ps3 += p3;
            cv.h[i >> 1] = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
            cv.h[8 + (i >> 1)] = __builtin_convertvector((f32x2){p2, p3}, bf16x2);
        }
        return (ps0 + ps1) + (ps2 + ps3);
    };
    auto vphase = [&](int t) {
        const int kt = kt0 + t;
        const bool plain = t > 0 && kt * BN + BN - 1 <= wave_vis_min;   // every key visible to every row, m is set
        float pt = 0.f;
        bool redo = !plain;
        if (plain) {
            // No maximum is taken: the row sums, needed anyway, show when a row has outgrown its reference
            // (32 numerators summing above 32 * 2^kLazy, or an overflow of exp2); only then the slow way.
            pt = numerators(m);
            redo = __builtin_amdgcn_ballot_w64(!(pt <= kSumCap)) != 0;
        }
        if (redo) {
            if (!plain) {
                int jb = kt * BN + 8 * jh;
                asm volatile("" : "+v"(jb));           // (made here: sixteen key offsets kept in registers across the tile loop cost more)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = jb + 16 * (i >> 3) + (i & 7);
                    if (key > vis) sa[i] = -INFINITY;
                    if (key + 32 > vis) sb[i] = -INFINITY;
                }
            }
            float mx = fmaxf(sa[0], sb[0]);            // the chain's first read of both accumulators
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = max3(mx, sa[i], sb[i]);
            {
                auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            }
            const float mxs = mx * sl2;
            const bool grow = mxs > m + kLazy;         // also true for a first visible key (m = -inf)
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float mn = grow ? mxs : m;
                const float alpha = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mn);   // o and l are 0 then
                l *= alpha;
                m = mn;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) o[dt] *= alpha;
            }
            // a row that has seen no key yet still has m = -inf and only -inf scores: keep inf - inf out
            pt = numerators(m == -INFINITY ? 0.f : m);
        }
        l += pt;
    };

#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks].v));   // q landed before the loop

    const bool last_is_tail = (kt0 + nt) * BN > ctx;   // the item's last key tile reaches past the context
    using T1 = std::integral_constant<bool, true>;
    using T0 = std::integral_constant<bool, false>;

    // F8, prologue: this lane's pieces of stage t -> bf16, outside a matrix phase
    auto widen = [&](int t) {
        const unsigned char* src = &land[F8 ? t % NSTAGE : 0][0] + w_src;
        unsigned char* dst = &ring[t % NSTAGE][0];
        Frag lo, hi;
        fp8x16_to_bf16(*(const uint4*)src, lo, hi);
        *(uint4*)(dst + w_dst_k) = lo.u;
        *(uint4*)(dst + (w_dst_k ^ 16)) = hi.u;
        fp8x16_to_bf16(*(const uint4*)(src + LAND_V), lo, hi);
        *(uint4*)(dst + w_dst_v) = lo.u;
        *(uint4*)(dst + (w_dst_v ^ 16)) = hi.u;
        __builtin_amdgcn_s_waitcnt(0xc07f);            // lgkmcnt(0): read, before the slot is requested again; written
    };

    // Both groups walk the same list of phases; group 1 does it one barrier later.
    // bf16: stage s is complete (every wave's part landed) at barrier b(2s - 1), one phase before group
    // 0's M(s), so that both groups can prefetch from it in the vector phase before their M(s).
    // F8: a wave keeps three stages of codes in flight; it requests a stage as soon as it has widened the
    // stage three before it.  Here: stages 0 and 1 (waves 4-7: and 2), the rest in the matrix phases.
    if constexpr (F8) {
        landed(0);
        widen(0);
        if (nt >= 3) issue();                          // stage 3
        landed(min(1, nt));
        widen(1);                                      // (stage 1 always exists: nt >= 1)
        if (group == 1) {
            if (nt >= 4) issue();                      // stage 4
            if (nt >= 2) { landed(2); widen(2); }
            __builtin_amdgcn_s_barrier();              // b0
        }
        __builtin_amdgcn_s_barrier();                  // b0 (group 0) / b1 (group 1): stages 0 and 1 are bf16
    } else {
        if (group == 1) {
            landed(1 < nt ? 1 : nt);                   // its parts of stages 0 and 1
            __builtin_amdgcn_s_barrier();              // b0
        }
        landed(0);
        __builtin_amdgcn_s_barrier();                  // b0 (group 0) / b1 (group 1)
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
    mphase(0, T0{}, T1{});
    __builtin_amdgcn_s_setprio(0);
    if (!F8 && group == 0) landed(min(1, nt));         // group 0 arrives at b1: stage 1
    // vector phase of key tile t between two barriers; requests stage t + 4 when `more`
    auto vector_part = [&](int t, bool prefetch) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();                  // b(2t + 1) / b(2t + 2)
        __builtin_amdgcn_sched_barrier(0);
        // M(t) of both groups is over once group 1 is here; group 0 learns that one barrier later
        if (group == 1 && (int)next_t <= nt) issue();       // stage t + 4 (F8: t + 5)
        if (prefetch) prefetch_v(t + 1);
        vphase(t);
        if (!F8 && group == 1) landed(min(t + 2, nt));  // bf16: group 1 arrives at b(2t + 3): stage t + 2
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();                  // b(2t + 2) / b(2t + 3)
        __builtin_amdgcn_sched_barrier(0);
        if (group == 0 && (int)next_t <= nt) issue();       // stage t + 4
        if (F8) landed(min(t + 2 + group, nt));        // F8: the codes this wave widens in the matrix phase that follows
    };
    for (int t = 0; t + 1 < nt; ++t) {
        vector_part(t, true);
        __builtin_amdgcn_s_setprio(1);
        mphase(t + 1, T1{}, T1{});
        __builtin_amdgcn_s_setprio(0);
        if (F8) __builtin_amdgcn_s_waitcnt(0xc07f);    // lgkmcnt(0): the widened pieces are written
        else if (group == 0) landed(min(t + 2, nt));   // group 0 arrives at b(2t + 3): stage t + 2
    }
    // the last key tile: its vector phase, then M(nt) = its PV
    vector_part(nt - 1, !last_is_tail);
    if (last_is_tail) pv_tail(nt);
    else mphase(nt, T1{}, T0{});
    if (group == 0) __builtin_amdgcn_s_barrier();      // b(2 nt + 1)
    KUN_WAIT_VMCNT(0);                                 // (nothing is in flight any more; no load may outlive the item)

    const float lt = l + __shfl_xor(l, 32);
    if (part_slot >= 0) {
        const size_t wg_rec = (size_t)part_slot * a.Hkv + kvh;
        float* po = a.part_o + wg_rec * (D * kSplitRows) + wave * ROWS_W + n;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) po[(32 * dt + 8 * (i >> 2) + 4 * jh + (i & 3)) * kSplitRows] = o[dt][i];
        if (jh == 0) *(float2*)(a.part_ml + (wg_rec * kSplitRows + wave * ROWS_W + n) * 2) = make_float2(m, lt);
    }
    const float inv = 1.0f / lt;
    if (live_row && part_slot < 0) {
        char* orow = (char*)a.out + (((size_t)(qs + pos)) * a.Hq + kvh * G + g_head) * (D * 2);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int dim = 32 * dt + 8 * i4 + 4 * jh;
                union { bf16x2 h[2]; uint2 u; } w;
                w.h[0] = __builtin_convertvector((f32x2){o[dt][4 * i4 + 0] * inv, o[dt][4 * i4 + 1] * inv}, bf16x2);
                w.h[1] = __builtin_convertvector((f32x2){o[dt][4 * i4 + 2] * inv, o[dt][4 * i4 + 3] * inv}, bf16x2);
                *(uint2*)(orow + dim * 2) = w.u;
            }
    }
    if (!PERSIST) return;
    }
}


// Rows of a split item from the partial results of its key ranges: m = max m_i, l = sum l_i 2^(m_i - m),
// o = sum o_i 2^(m_i - m) / l.  One workgroup per (split item, kv head, 16 dims), one thread per row.
constexpr int kMergeDims = 16;
__global__ __launch_bounds__(kSplitRows) void prefill_merge_kernel(const PrefillArgs a, int G) {
    constexpr int NDC = D / kMergeDims;
    const int dc = blockIdx.x % NDC;
    const int si = blockIdx.x / NDC / a.Hkv, kvh = blockIdx.x / NDC % a.Hkv;
    if (a.n_items[1] != a.plan_tag || si >= *a.n_split_items) return;
    const int4 it = a.split_items[si];
    const int chunk = it.x, qt = it.y, nsplit = it.z, slot0 = it.w;
    const int qs = a.q_start[chunk];
    const int c = a.q_start[chunk + 1] - qs;
    const int row = threadIdx.x;
    const int pos = qt * (kSplitRows / G) + row / G, head = row % G;
    if (row >= kSplitRows / G * G || pos >= c) return;      // (the workgroup's last rows are dead when G does not divide 256)
    float w[kMaxSplit];
    float M = -INFINITY;
    for (int sp = 0; sp < nsplit; ++sp)
        M = fmaxf(M, a.part_ml[((((size_t)slot0 + sp) * a.Hkv + kvh) * kSplitRows + row) * 2]);
    float l = 0.f;
#pragma unroll
    for (int sp = 0; sp < kMaxSplit; ++sp) {
        w[sp] = 0.f;
        if (sp < nsplit) {
            const size_t rec = (((size_t)slot0 + sp) * a.Hkv + kvh) * kSplitRows + row;
            const float mi = a.part_ml[rec * 2];
            w[sp] = (mi == -INFINITY) ? 0.f : exp2f(mi - M);      // -inf: the row sees no key of this range
            l += w[sp] * a.part_ml[rec * 2 + 1];
        }
    }
    const float inv = 1.0f / l;
    char* orow = (char*)a.out + (((size_t)(qs + pos)) * a.Hq + kvh * G + head) * (D * 2);
    for (int d0 = dc * kMergeDims; d0 < (dc + 1) * kMergeDims; d0 += 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sp = 0; sp < kMaxSplit; ++sp) {
            if (sp < nsplit) {
                const float* po = a.part_o + (((size_t)slot0 + sp) * a.Hkv + kvh) * (D * kSplitRows) + row;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += w[sp] * po[(d0 + e) * kSplitRows];
            }
        }
        union { bf16x2 h[4]; uint4 u; } v;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            v.h[e] = __builtin_convertvector((f32x2){acc[2 * e] * inv, acc[2 * e + 1] * inv}, bf16x2);
        *(uint4*)(orow + d0 * 2) = v.u;
    }
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Shapes the MFMA kernels do not cover (fp32, head_dim 64): row r of chunk i is the decode of a
// request of p_i + r + 1 tokens behind table row i.
// Every query row looks its chunk up (q_start ascends; a row that no consistent chunk covers gets
// length 0 and is skipped like an empty request), so each entry is written exactly once.
__global__ __launch_bounds__(256) void prefill_rows_kernel(const int32_t* __restrict__ q_start,
                                                           const int32_t* __restrict__ prior, int n_chunks,
                                                           int total_new, long long row_tokens,
                                                           int32_t* __restrict__ ctx_len,
                                                           int32_t* __restrict__ row_of_seq) {
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < total_new; t += gridDim.x * blockDim.x) {
        int lo = 0, hi = n_chunks;                         // last chunk that starts at or before row t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (q_start[mid] <= t) lo = mid; else hi = mid;
        }
        int len = 0;
        if (n_chunks > 0) {
            const int c = chunk_tokens(q_start, prior, lo, total_new, row_tokens);
            const int r = t - q_start[lo];
            if (c > 0 && r >= 0 && r < c) len = prior[lo] + r + 1;
        }
        ctx_len[t] = len;
        row_of_seq[t] = lo;
    }
}

bool mfma_shape(const kun_kv_pool* p) { return (p->dtype == KUN_BF16 || p->dtype == KUN_FP8_E4M3) && p->d == 128; }

// compute units of the current device (one fetching workgroup each)
int device_compute_units() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    return n;
}

template <int G>
void launch_tiles(const PrefillArgs& a, dim3 grid, bool persistent, bool ring, bool fp8, hipStream_t st) {
    if (fp8) {
        if (persistent) hipLaunchKernelGGL((prefill_pp_kernel<G, true, true>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((prefill_pp_kernel<G, false, true>), grid, dim3(512), 0, st, a);
    } else if (ring) {
        if (persistent) hipLaunchKernelGGL((prefill_ring_kernel<G, true>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((prefill_ring_kernel<G, false>), grid, dim3(512), 0, st, a);
    } else {
        if (persistent) hipLaunchKernelGGL((prefill_pp_kernel<G, true, false>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((prefill_pp_kernel<G, false, false>), grid, dim3(512), 0, st, a);
    }
}

bool prefill_shape_ok(const kun_kv_pool* p, int n_chunks, int Hq, int total_new, int max_blocks) {
    return p && n_chunks >= 0 && Hq > 0 && Hq % p->Hkv == 0 && total_new >= 0 && max_blocks >= 0;
}

int sub_shift_of(const kun_kv_pool* p) { return p->B == 128 ? 3 : p->B == 64 ? 2 : p->B == 32 ? 1 : 0; }

// Workspace of the MFMA path: header (256 B: n_items, the 8 fetch counters at +64, n_split_items at
// +128), the item list and its descriptors, the resolved address of every 16-token page tile of every
// chunk, and -- only when the launch is small enough to be split -- the per-item split records, the
// list of split items and the partial results of the key ranges.
struct PrefillLayout {
    bool may_split;
    int max_items, cap_entries;
    size_t off_items, off_desc, off_pages, off_split_info, off_split_items, off_part_ml, off_part_o, total;
};

PrefillLayout prefill_layout(const kun_kv_pool* p, int n_chunks, int Hq, int total_new_tokens, int max_blocks) {
    PrefillLayout lay;
    const int G = Hq / p->Hkv;
    const int pos_per_tile = kSplitRows / G;               // whole query positions per workgroup
    // at least total / pos items exist, so a launch with that many workgroups or more is never split
    lay.may_split = (int64_t)(total_new_tokens / pos_per_tile) * p->Hkv < kSplitTarget;
    lay.max_items = total_new_tokens / pos_per_tile + n_chunks;
    lay.cap_entries = lay.may_split ? 2 * lay.max_items + kSplitTarget / p->Hkv + 1 : lay.max_items;
    size_t o = 256;
    lay.off_items = o;        o += align256(sizeof(int2) * (size_t)lay.cap_entries);
    lay.off_desc = o;         o += align256(sizeof(int4) * 2 * (size_t)lay.cap_entries);
    lay.off_pages = o;        o += align256(sizeof(unsigned long long) * (size_t)n_chunks * (size_t)page_row_entries(max_blocks, sub_shift_of(p)));
    lay.off_split_info = o;   if (lay.may_split) o += align256(sizeof(int2) * (size_t)lay.cap_entries);
    lay.off_split_items = o;  if (lay.may_split) o += align256(sizeof(int4) * (size_t)(kSplitTarget + 1));
    const size_t part_wgs = 2 * (size_t)kSplitTarget + p->Hkv;       // (key range, kv head) workgroups of split items
    lay.off_part_ml = o;      if (lay.may_split) o += align256(sizeof(float) * 2 * kSplitRows * part_wgs);
    lay.off_part_o = o;       if (lay.may_split) o += align256(sizeof(float) * D * kSplitRows * part_wgs);
    lay.total = o;
    return lay;
}

}  // namespace

extern "C" size_t kun_prefill_workspace_bytes(const kun_kv_pool* p, int n_chunks, int Hq, int total_new_tokens,
                                              int max_blocks) {
    if (!prefill_shape_ok(p, n_chunks, Hq, total_new_tokens, max_blocks)) return 0;
    if (!mfma_shape(p))                                    // rows as decode requests: two int32 per row + its plan
        return 256 + 2 * align256(sizeof(int32_t) * (size_t)total_new_tokens) +
               kun_attend_rows_workspace_bytes(total_new_tokens);
    const int G = Hq / p->Hkv;
    if (G < 1 || (G > 8 && G != 16)) return 0;
    return prefill_layout(p, n_chunks, Hq, total_new_tokens, max_blocks).total;
}

namespace {

// max_workgroups == 0: one workgroup per work item (or, with the option "persistent", one fetching
// workgroup per compute unit); otherwise that many workgroups (rounded down to a multiple of 8, at
// least 8) fetch the items.
// steps: the plan launch and the rest (kPlanAndRun), or one of the two.
enum PrefillSteps { kPlanAndRun = 0, kPlanOnly = 1, kRunOnly = 2 };

// What identifies the plan a call expects to find in its workspace (never 0).
int prefill_plan_tag(int n_chunks, int total_new_tokens, int max_blocks, int Hkv, int G, int sub_shift) {
    uint32_t h = 0x85ebca6bu;
    for (uint32_t v : {(uint32_t)n_chunks, (uint32_t)total_new_tokens, (uint32_t)max_blocks, (uint32_t)Hkv, (uint32_t)G,
                       (uint32_t)sub_shift}) {
        h ^= v + 0x9e3779b9u + (h << 6) + (h >> 2);
    }
    return (int)(h | 1u);
}

int prefill_enqueue(kun_kv_pool* p, const void* q, void* out, const int32_t* q_start, const int32_t* prior_len,
                    const int32_t* block_table, int max_blocks, int n_chunks, int Hq, int total_new_tokens,
                    float scale, int max_workgroups, void* workspace, size_t workspace_bytes, void* stream,
                    PrefillSteps steps = kPlanAndRun) {
    if (!prefill_shape_ok(p, n_chunks, Hq, total_new_tokens, max_blocks) || max_workgroups < 0) return KUN_ERR_INVALID_ARG;
    if (n_chunks == 0 || total_new_tokens == 0) return KUN_OK;
    if (!q_start || !prior_len || !block_table || max_blocks <= 0) return KUN_ERR_INVALID_ARG;
    if (steps != kPlanOnly && (!q || !out)) return KUN_ERR_INVALID_ARG;
    const int G = Hq / p->Hkv;
    if (G < 1 || (G > 8 && !(G == 16 && mfma_shape(p)))) return KUN_ERR_UNSUPPORTED;   // 16: the MFMA kernels only
    const size_t need = kun_prefill_workspace_bytes(p, n_chunks, Hq, total_new_tokens, max_blocks);
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < need) return KUN_ERR_WORKSPACE;
    if (!mfma_shape(p)) {
        if (steps == kPlanOnly) return KUN_OK;             // (row by row: the rows' list is made by the call itself)
        const size_t col = align256(sizeof(int32_t) * (size_t)total_new_tokens);
        int32_t* ctx_len = (int32_t*)((char*)workspace + 256);
        int32_t* row_of_seq = (int32_t*)((char*)workspace + 256 + col);
        hipStream_t st = (hipStream_t)stream;
        const int row_wgs = (total_new_tokens + 255) / 256;
        hipLaunchKernelGGL(prefill_rows_kernel, dim3((unsigned)(row_wgs < 4096 ? row_wgs : 4096)), dim3(256), 0, st,
                           q_start, prior_len, n_chunks, total_new_tokens, (long long)max_blocks * p->B, ctx_len,
                           row_of_seq);
        KUN_HIP_CHECK_LAUNCH();
        return kun_attend_rows_generic(p, q, out, block_table, max_blocks, ctx_len, row_of_seq, total_new_tokens, Hq,
                                       scale, (char*)workspace + 256 + 2 * col, st);
    }

    // (fetching workgroups count through the list with counters that only the plan launch clears)
    bool persistent = steps == kPlanAndRun &&
                      (max_workgroups > 0 || kun_options().prefill_shape == 1 || kun_options().prefill_shape == 3);
    if (persistent && max_workgroups == 0) max_workgroups = device_compute_units();
    const int pos_per_tile = kSplitRows / G;
    const PrefillLayout lay = prefill_layout(p, n_chunks, Hq, total_new_tokens, max_blocks);
    const bool can_split = lay.may_split;
    char* ws = (char*)workspace;
    PrefillArgs a;
    a.rt = p->ranges;
    a.q = q;
    a.out = out;
    a.q_start = q_start;
    a.prior = prior_len;
    a.table = block_table;
    a.n_items = (int32_t*)ws;
    a.next_item = (int32_t*)ws + 16;
    a.n_split_items = (int32_t*)ws + 32;
    a.items = (int2*)(ws + lay.off_items);
    a.desc = (const int4*)(ws + lay.off_desc);
    a.page_addr = (const unsigned long long*)(ws + lay.off_pages);
    a.tiles_per_row = page_row_entries(max_blocks, sub_shift_of(p));
    a.split_info = can_split ? (const int2*)(ws + lay.off_split_info) : nullptr;
    a.split_items = (int4*)(ws + lay.off_split_items);
    a.part_ml = (float*)(ws + lay.off_part_ml);
    a.part_o = (float*)(ws + lay.off_part_o);
    a.max_blocks = max_blocks;
    a.n_chunks = n_chunks;
    a.Hkv = p->Hkv;
    a.Hq = Hq;
    a.max_items = lay.max_items;
    a.scale_log2 = scale * kLog2e;
    a.block_bytes = (unsigned)p->block_bytes;
    a.page_bytes = (unsigned)p->page_bytes;
    a.sub_shift = sub_shift_of(p);
    hipStream_t st = (hipStream_t)stream;

    // one launch: workgroup 0 makes the work list, the others resolve the blocks of every chunk
    ResolveArgs ra;
    ra.rt = p->ranges;
    ra.table = block_table;
    ra.page_addr = (unsigned long long*)(ws + lay.off_pages);
    ra.max_blocks = max_blocks;
    ra.total_new = total_new_tokens;
    ra.last_block = p->ranges.first[p->ranges.n] - 1;
    ra.sub_shift = a.sub_shift;
    ra.block_bytes = a.block_bytes;
    ra.tile_bytes = (unsigned)(2 * kBlock * D * p->elt);
    const size_t n_entries = (size_t)n_chunks * (size_t)a.tiles_per_row;
    ra.n_wgs = (int)((n_entries + kPlanThreads - 1) / kPlanThreads < 1024 ? (n_entries + kPlanThreads - 1) / kPlanThreads : 1024);
    a.plan_tag = prefill_plan_tag(n_chunks, total_new_tokens, max_blocks, p->Hkv, G, a.sub_shift);
    if (steps != kRunOnly) {
        hipLaunchKernelGGL(prefill_plan_kernel, dim3(1 + ra.n_wgs), dim3(kPlanThreads), 0, st, ra, q_start, prior_len,
                           n_chunks, pos_per_tile, a.max_items, a.n_items, a.next_item, a.items, p->Hkv,
                           can_split ? kSplitTarget : 0, lay.cap_entries, (int2*)(ws + lay.off_split_info),
                           a.split_items, a.n_split_items, (int4*)(ws + lay.off_desc), a.plan_tag);
        KUN_HIP_CHECK_LAUNCH();
    }
    if (steps == kPlanOnly) return KUN_OK;
    size_t wgs = (size_t)(can_split ? lay.cap_entries : lay.max_items) * p->Hkv;
    if (persistent) {
        const size_t lim = max_workgroups < 8 ? 8 : (size_t)(max_workgroups & ~7);
        if (wgs > lim) wgs = lim;
        wgs = (wgs + 7) & ~(size_t)7;                  // every residue class mod 8 needs a workgroup
    }
    const dim3 grid((unsigned)wgs);
    const bool ring = kun_options().prefill_shape >= 2;     // the one-barrier-per-tile kernel (cross-check)
    switch (G) {
        case 1: launch_tiles<1>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
        case 2: launch_tiles<2>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
        case 3: launch_tiles<3>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
        case 4: launch_tiles<4>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
        case 5: launch_tiles<5>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
        case 6: launch_tiles<6>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
        case 7: launch_tiles<7>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
        case 8: launch_tiles<8>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
        default: launch_tiles<16>(a, grid, persistent, ring, p->dtype == KUN_FP8_E4M3, st); break;
    }
    KUN_HIP_CHECK_LAUNCH();
    if (can_split) {
        hipLaunchKernelGGL(prefill_merge_kernel,
                           dim3((unsigned)((kSplitTarget / p->Hkv + 1) * p->Hkv * (D / kMergeDims))), dim3(kSplitRows), 0,
                           st, a, G);
        KUN_HIP_CHECK_LAUNCH();
    }
    return KUN_OK;
}

}  // namespace

extern "C" int kun_paged_prefill_chunk(kun_kv_pool* p, const void* q, void* out, const int32_t* q_start,
                                       const int32_t* prior_len, const int32_t* block_table, int max_blocks,
                                       int n_chunks, int Hq, int total_new_tokens, float scale,
                                       void* workspace, size_t workspace_bytes, void* stream) {
    return prefill_enqueue(p, q, out, q_start, prior_len, block_table, max_blocks, n_chunks, Hq, total_new_tokens,
                           scale, 0, workspace, workspace_bytes, stream);
}

extern "C" int kun_prefill_plan(kun_kv_pool* p, const int32_t* q_start, const int32_t* prior_len,
                               const int32_t* block_table, int max_blocks, int n_chunks, int Hq,
                               int total_new_tokens, void* workspace, size_t workspace_bytes, void* stream) {
    return prefill_enqueue(p, nullptr, nullptr, q_start, prior_len, block_table, max_blocks, n_chunks, Hq,
                           total_new_tokens, 1.0f, 0, workspace, workspace_bytes, stream, kPlanOnly);
}

extern "C" int kun_paged_prefill_chunk_planned(kun_kv_pool* p, const void* q, void* out, const int32_t* q_start,
                                               const int32_t* prior_len, const int32_t* block_table, int max_blocks,
                                               int n_chunks, int Hq, int total_new_tokens, float scale,
                                               void* workspace, size_t workspace_bytes, void* stream) {
    return prefill_enqueue(p, q, out, q_start, prior_len, block_table, max_blocks, n_chunks, Hq, total_new_tokens,
                           scale, 0, workspace, workspace_bytes, stream, kRunOnly);
}

extern "C" int kun_paged_prefill_chunk_on(kun_kv_pool* p, const void* q, void* out, const int32_t* q_start,
                                          const int32_t* prior_len, const int32_t* block_table, int max_blocks,
                                          int n_chunks, int Hq, int total_new_tokens, float scale,
                                          int max_workgroups, void* workspace, size_t workspace_bytes,
                                          void* stream) {
    if (max_workgroups <= 0) return KUN_ERR_INVALID_ARG;
    return prefill_enqueue(p, q, out, q_start, prior_len, block_table, max_blocks, n_chunks, Hq, total_new_tokens,
                           scale, max_workgroups, workspace, workspace_bytes, stream);
}
