// Batched paged decode: split-K over the KV blocks of each request, then a merge of the partial
// results.  Decode streams the whole KVCache of every request once and is memory-bound
// (Section 2.1); after a parameter drop the batch and the pool are larger (Section 3), so this is
// the kernel whose time grows with the pool.
//
// Launch sequence (one stream, no host synchronisation):
//   1. plan     -- one workgroup turns ctx_len[] into a list of work items (request, partition)
//                  of `part_tokens` tokens each and a per-request index of its first item, and
//                  clears the arrival counters.
//   2. partial  -- one workgroup per (item, kv head): online softmax over the item's tokens for
//                  the G query heads that share the kv head, K/V pages read exactly once.
//                  Requests that fit one partition are normalised and written to `out` directly;
//                  otherwise the workgroup writes a partial record.
//   3. merge    -- o = sum_i acc_i e^(m_i - M) / sum_i l_i e^(m_i - M), records in partition order.
//                  Small batches: inside the partial kernel, by the LAST workgroup of a (request,
//                  kv head) to arrive (one device-scope counter per pair).  Large batches: a launch
//                  of its own, one workgroup group per (request, kv head) with several partitions.
//
// Two partial kernels: a generic one on the vector ALUs (any supported dtype/shape; used for
// fp32) and an MFMA one for bf16 with head_dim 128, where the G query rows are padded to a
// 16-wide MFMA tile so that the inner products cost almost nothing next to the page loads.
#include <math.h>
#include <stdlib.h>

#include <mutex>
#include <type_traits>

#include "kun_internal.h"

namespace {

constexpr int kBlock = 16;           // tokens per page tile: a 16-token block, or one of the four tiles of a 64-token block
constexpr float kLog2e = 1.4426950408889634f;

struct DecodeArgs {
    KunRanges rt;
    const void* q;
    void* out;
    const int32_t* table;
    const int32_t* ctx_len;
    const int32_t* row_of_seq;  // optional: block-table row of each request (NULL: request s uses row s)
    int32_t* n_items;        // workspace: number of work items (written by plan)
    int32_t* seq_first;      // workspace: [S + 1] first item of each request
    int4* items;             // workspace: (request, partition, the request's context length, record slot)
    int32_t* arrived;        // workspace: [S, Hkv] partitions of a (request, kv head) whose records are written
    float* part_ml;          // workspace: [item, kvh, G, 2]  (m in log2 units, l)
    float* part_acc;         // workspace: [item, kvh, G, d]
    int max_blocks;
    int S, Hkv, G;
    int last_block;          // largest block id of the pool: table entries are clamped into [0, last_block] before they
                             // become addresses, so that a bad entry reads some block of the pool, never anything else
    int B;                   // tokens per KV block: 16, 32, 64 or 128
    int tile_shift;          // log2(B / 16)
    int part_tokens;         // tokens per partition, multiple of 32
    int max_items;
    float scale_log2;        // softmax scale * log2(e)
    unsigned block_bytes, page_bytes;
    int xcd_map;             // MFMA kernel: the KV heads of a work item run on one XCD
    int fold;                // the last workgroup of a (request, kv head) merges its records (else decode_merge_kernel does)
    int plan_tag;            // what the plan launch left behind n_items: a call on a workspace that holds no plan for
                             // this batch shape (kun_paged_decode_planned without its plan) computes nothing
};

// The header of the workspace: list length, tag of the plan that wrote it.
struct PlanHeader { int n_items, tag; };
__device__ __forceinline__ PlanHeader load_plan_header(const DecodeArgs& a) {
    const int2 h = *(const int2*)a.n_items;
    return PlanHeader{h.x, h.y};
}

// ---------------------------------------------------------------------------------------------
// 1. plan
// ---------------------------------------------------------------------------------------------
// Record slots (where a partition's partial result goes) count through the requests in order:
// request s owns slots seq_first[s] .. seq_first[s + 1] - 1.  The work list is ordered for the
// launch instead: first every full partition (all the same length), then the requests' last,
// shorter partitions from long to short (counting sort over kLenBuckets length classes), so that
// the workgroups that start last are the shortest ones.  An entry is (request, partition, context
// length, record slot).
constexpr int kLenBuckets = 32;
__global__ __launch_bounds__(1024) void decode_plan_kernel(const int32_t* __restrict__ ctx_len, int S,
                                                         int part_tokens, int max_items,
                                                         int32_t* __restrict__ n_items,
                                                         int32_t* __restrict__ seq_first,
                                                         int4* __restrict__ items,
                                                         int32_t* __restrict__ arrived, int n_arrived, int tag) {
    for (int i = threadIdx.x; i < n_arrived; i += 1024) arrived[i] = 0;
    if (threadIdx.x == 0) n_items[1] = tag;
    __shared__ int wave_tot[16], wave_full[16];
    __shared__ int carry_s, carry_full;
    __shared__ int bucket[kLenBuckets];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { carry_s = 0; carry_full = 0; }
    if (tid < kLenBuckets) bucket[tid] = 0;
    __syncthreads();
    for (int s0 = 0; s0 < S; s0 += 1024) {
        const int s = s0 + tid;
        int np = 0, nfull = 0, L = 0;
        if (s < S) {
            L = ctx_len[s];
            if (L < 0) L = 0;
            nfull = L / part_tokens;
            np = (L + part_tokens - 1) / part_tokens;
        }
        int incl = np, incl_f = nfull;       // inclusive scans inside the wave
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o), yf = __shfl_up(incl_f, o);
            if (lane >= o) { incl += y; incl_f += yf; }
        }
        if (lane == 63) { wave_tot[wave] = incl; wave_full[wave] = incl_f; }
        __syncthreads();
        int before = carry_s, before_f = carry_full;
        for (int w = 0; w < wave; ++w) { before += wave_tot[w]; before_f += wave_full[w]; }
        const int first = before + incl - np, first_f = before_f + incl_f - nfull;
        if (s < S) {
            seq_first[s] = first;
            for (int p = 0; p < nfull; ++p)
                if (first_f + p < max_items) items[first_f + p] = make_int4(s, p, L, first + p);
            if (np > nfull) atomicAdd(&bucket[(part_tokens - (L - nfull * part_tokens)) * kLenBuckets / part_tokens], 1);
        }
        __syncthreads();
        if (tid == 1023) { carry_s = first + np; carry_full = first_f + nfull; }
        __syncthreads();
    }
    if (tid == 0) {
        int at = carry_full;                 // the shorter partitions follow the full ones, bucket 0 (longest) first
        for (int b = 0; b < kLenBuckets; ++b) {
            const int n = bucket[b];
            bucket[b] = at;
            at += n;
        }
        const int tot = carry_s;
        seq_first[S] = tot;
        *n_items = tot < max_items ? tot : max_items;
    }
    __syncthreads();
    if (carry_s > max_items) {
        // More partitions than the caller's bound allows for: list position = record slot, in request
        // order, so that exactly the requests whose slots all fit are computed, and completely.
        for (int s = tid; s < S; s += 1024) {
            const int L = ctx_len[s], first = seq_first[s];
            const int np = L > 0 ? (L + part_tokens - 1) / part_tokens : 0;
            for (int p = 0; p < np && first + p < max_items; ++p)
                items[first + p] = make_int4(s, p, L, first + np <= max_items ? first + p : max_items);
        }
        return;
    }
    for (int s = tid; s < S; s += 1024) {
        const int L = ctx_len[s];
        if (L <= 0) continue;
        const int nfull = L / part_tokens, rem = L - nfull * part_tokens;
        if (rem == 0) continue;
        const int pos = atomicAdd(&bucket[(part_tokens - rem) * kLenBuckets / part_tokens], 1);
        items[pos] = make_int4(s, nfull, L, seq_first[s] + nfull);
    }
}

// ---------------------------------------------------------------------------------------------
// helpers
// ---------------------------------------------------------------------------------------------
// 16-byte load of K/V page data, which a decode step reads exactly once: marked non-temporal so that
// it streams past the caches (measured on a plain read of a 16 GiB buffer: 7.0 TB/s against 6.2 TB/s
// for ordinary loads).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// The pointer is cast to the global address space: a load through a generic pointer is a flat load,
// which may complete out of order with other loads, so every wait for one waits for all of them.
__device__ __forceinline__ uint4 load_stream16(const void* p) {
    const u32x4 v = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) {
    return __uint_as_float((unsigned)b << 16);
}
__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerLoad = 4;   // elements per 16-byte load
    __device__ static float get(const uint4& v, int i) {
        return __uint_as_float(i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w);
    }
    __device__ static void store(float* p, float x) { *p = x; }
};
struct bf16_t { unsigned short bits; };
template <> struct Elem<bf16_t> {
    static constexpr int kPerLoad = 8;
    __device__ static float get(const uint4& v, int i) {
        unsigned w = (i >> 1) == 0 ? v.x : (i >> 1) == 1 ? v.y : (i >> 1) == 2 ? v.z : v.w;
        return (i & 1) ? __uint_as_float(w & 0xffff0000u) : __uint_as_float(w << 16);
    }
    __device__ static void store(bf16_t* p, float x) { p->bits = f32_to_bf16_rne(x); }
};

// K/V pages as OCP FP8 E4M3 codes (1 sign, 4 exponent, 3 mantissa bits; bias 7): converted exactly by the
// hardware's conversion instruction.  Queries and outputs of such pools are bf16.
struct fp8_t { unsigned char bits; };
template <> struct Elem<fp8_t> {
    static constexpr int kPerLoad = 16;
    __device__ static float get(const uint4& v, int i) {
        const unsigned w = (i >> 2) == 0 ? v.x : (i >> 2) == 1 ? v.y : (i >> 2) == 2 ? v.z : v.w;
        switch (i & 3) {
            case 0: return __builtin_amdgcn_cvt_f32_fp8(w, 0);
            case 1: return __builtin_amdgcn_cvt_f32_fp8(w, 1);
            case 2: return __builtin_amdgcn_cvt_f32_fp8(w, 2);
            default: return __builtin_amdgcn_cvt_f32_fp8(w, 3);
        }
    }
};
// element type of queries and outputs for pages of type T
template <typename T> struct QueryOf { typedef T type; };
template <> struct QueryOf<fp8_t> { typedef bf16_t type; };

// Stores and loads of partial records that are coherent across the whole device (they bypass what
// the XCD-local L2 may hold of the line): relaxed atomic accesses at device scope.
__device__ __forceinline__ void rec_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float rec_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// out[seq, heads of kvh] from the nparts partial records that start at record slot `first`: the records
// are combined in partition order, two per step, whoever does it, so the result does not depend on
// which workgroup merges or when.  Elements idx0, idx0 + stride, ... of the G x D outputs.
template <typename T, int D, bool COHERENT>
__device__ __forceinline__ void merge_records(const DecodeArgs& a, int first, int nparts, int kvh, int seq, int G,
                                              int idx0, int stride) {
    auto ld = [](const float* p) { return COHERENT ? rec_load(p) : *p; };
    for (int idx = idx0; idx < G * D; idx += stride) {
        const int g = idx / D, j = idx - g * D;
        const size_t rec0 = (((size_t)first) * a.Hkv + kvh) * G + g, step = (size_t)a.Hkv * G;
        float M = -INFINITY;
        for (int p = 0; p < nparts; ++p) M = fmaxf(M, ld(&a.part_ml[(rec0 + p * step) * 2]));
        float l = 0.f, acc = 0.f;
        int p = 0;
        for (; p + 1 < nparts; p += 2) {                   // two independent records per step
            const size_t r0 = rec0 + p * step, r1 = r0 + step;
            const float m0 = ld(&a.part_ml[r0 * 2]), m1 = ld(&a.part_ml[r1 * 2]);
            const float l0 = ld(&a.part_ml[r0 * 2 + 1]), l1 = ld(&a.part_ml[r1 * 2 + 1]);
            const float a0 = ld(&a.part_acc[r0 * D + j]), a1 = ld(&a.part_acc[r1 * D + j]);
            const float f0 = exp2f(m0 - M), f1 = exp2f(m1 - M);
            l += f0 * l0;
            acc += f0 * a0;
            l += f1 * l1;
            acc += f1 * a1;
        }
        if (p < nparts) {
            const size_t r0 = rec0 + p * step;
            const float f0 = exp2f(ld(&a.part_ml[r0 * 2]) - M);
            l += f0 * ld(&a.part_ml[r0 * 2 + 1]);
            acc += f0 * ld(&a.part_acc[r0 * D + j]);
        }
        T* o = (T*)a.out + ((size_t)seq * a.Hkv * G + (size_t)kvh * G + g) * D + j;
        Elem<T>::store(o, acc / l);
    }
}

// Combine the per-wave partial results held in LDS and write either the final output row (request
// with one partition) or the item's partial record; the workgroup that completes the records of its
// (request, kv head) then merges them.  sm_m/sm_l: [NW][G]; sm_acc: [NW][G][D].  Called by every
// thread of the workgroup.
template <typename T, int D, int NW>
__device__ __forceinline__ void finish_item(const DecodeArgs& a, int slot, int part, int kvh, int seq, int nparts,
                                            int G, const float* sm_m, const float* sm_l,
                                            const float* sm_acc) {
    for (int idx = threadIdx.x; idx < G * D; idx += blockDim.x) {
        const int g = idx / D, j = idx - g * D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, sm_m[w * G + g]);
        float l = 0.f, acc = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = sm_m[w * G + g];
            const float f = (mw == -INFINITY) ? 0.f : exp2f(mw - M);
            l += f * sm_l[w * G + g];
            acc += f * sm_acc[(w * G + g) * D + j];
        }
        if (nparts == 1) {
            T* o = (T*)a.out + ((size_t)seq * a.Hkv * G + (size_t)kvh * G + g) * D + j;
            Elem<T>::store(o, acc / l);
        } else {
            const size_t rec = ((size_t)slot * a.Hkv + kvh) * G + g;
            if (a.fold) {
                rec_store(&a.part_acc[rec * D + j], acc);
                if (j == 0) {
                    rec_store(&a.part_ml[rec * 2 + 0], M);
                    rec_store(&a.part_ml[rec * 2 + 1], l);
                }
            } else {
                a.part_acc[rec * D + j] = acc;
                if (j == 0) {
                    a.part_ml[rec * 2 + 0] = M;
                    a.part_ml[rec * 2 + 1] = l;
                }
            }
        }
    }
    if (nparts == 1 || !a.fold) return;                  // (not folding: decode_merge_kernel follows)
    // The partitions of a request run on different XCDs, whose L2 caches do not see each other's
    // lines.  A device-wide fence would write back and invalidate a whole L2 per workgroup (measured:
    // the decode step took half as long again), so the records themselves go through device-coherent
    // stores and loads instead (rec_store / rec_load): every thread waits until its stores are
    // acknowledged, the workgroup meets at a barrier, and only then is its arrival counted; the
    // workgroup that counts the last arrival reads every record of the pair coherently.
    __shared__ int s_last;
    __builtin_amdgcn_s_waitcnt(0);                       // vmcnt(0): this thread's record stores are done
    __syncthreads();
    if (threadIdx.x == 0)
        s_last = __hip_atomic_fetch_add(&a.arrived[(size_t)seq * a.Hkv + kvh], 1, __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_AGENT) == nparts - 1;
    __syncthreads();
    if (!s_last) return;
    // Nobody else touches the counter any more: back to zero, so that a plan (which cleared the
    // counters once) serves any number of calls.
    if (threadIdx.x == 0)
        __hip_atomic_store(&a.arrived[(size_t)seq * a.Hkv + kvh], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    merge_records<T, D, true>(a, slot - part, nparts, kvh, seq, G, threadIdx.x, blockDim.x);
}

// ---------------------------------------------------------------------------------------------
// 2a. generic partial kernel (vector ALUs).  4 waves; each wave takes every 4th block.
//     Lane layout for K: LPR = D / EPL lanes cover one token row with one 16-byte load each, so a
//     load instruction covers TPL = 64 / LPR tokens.  For V^T ([D][16 tokens]) lane x owns dims
//     x, x + 64, ... and reads the 16 tokens of each.
// ---------------------------------------------------------------------------------------------
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_partial_generic(const DecodeArgs a) {
    constexpr int NW = 4;
    constexpr int EPL = Elem<T>::kPerLoad;
    constexpr int LPR = D / EPL;
    constexpr int TPL = 64 / LPR;
    constexpr int NIT = kBlock / TPL;
    constexpr int DPL = D / 64;                    // dims per lane in the PV phase
    constexpr int VLD = kBlock / EPL;              // 16-byte loads per V^T row
    __shared__ float sm_m[NW * G], sm_l[NW * G];
    __shared__ float sm_acc[NW * G * D];

    const int item = blockIdx.x / a.Hkv, kvh = blockIdx.x % a.Hkv;
    const PlanHeader hdr = load_plan_header(a);        // both loads go out together: the list is as long as the grid
    const int n_items = hdr.n_items;
    const int4 it4 = a.items[item];                    // the length rides along: one dependent load less
    if (hdr.tag != a.plan_tag || it4.z > (long long)a.max_blocks * a.B) return;   // no plan of this batch, or not of this table
    if (it4.z <= 0) return;                            // (a row list may hold rows without a context)
    if (item >= n_items || it4.w >= a.max_items) return;   // (a record slot beyond the workspace: the caller's bound was too small)
    const int seq = it4.x, part = it4.y;
    const int L = it4.z;
    const int nparts = (L + a.part_tokens - 1) / a.part_tokens;
    const int t0 = part * a.part_tokens;
    const int t1 = min(L, t0 + a.part_tokens);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane % LPR, grp = lane / LPR;

    typedef typename QueryOf<T>::type QT;              // queries and outputs
    constexpr int QPL = Elem<QT>::kPerLoad;            // query elements per 16-byte load
    float qf[G][EPL];
    {
        const QT* qrow = (const QT*)a.q + ((size_t)seq * a.Hkv + kvh) * G * D;
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int c = 0; c < EPL / QPL; ++c) {
                uint4 v = *(const uint4*)(qrow + g * D + col * EPL + c * QPL);
#pragma unroll
                for (int e = 0; e < QPL; ++e) qf[g][c * QPL + e] = Elem<QT>::get(v, e);
            }
    }
    float m[G], l[G], acc[G][DPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int i = 0; i < DPL; ++i) acc[g][i] = 0.f;
    }

    const int32_t* trow = a.table + (size_t)(a.row_of_seq ? a.row_of_seq[seq] : seq) * a.max_blocks;
    // b counts tiles of 16 tokens: tile b % (B / 16) of block b / (B / 16); a tile is K [16][D], then V^T [D][16]
    const int tiles_per_block = a.B / kBlock;
    for (int b = t0 / kBlock + wave; b * kBlock < t1; b += NW) {
        const int blk = min(max(__builtin_amdgcn_readfirstlane(trow[b / tiles_per_block]), 0), a.last_block);
        const char* page = kun_block_addr(a.rt, blk, a.block_bytes) + (size_t)kvh * a.page_bytes +
                           (size_t)(b % tiles_per_block) * (2 * kBlock * D * sizeof(T));
        const int tb = b * kBlock;
        // scores: s[g][it] for token tb + it * TPL + grp
        float s[G][NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int tok = it * TPL + grp;
            uint4 kv = load_stream16(page + ((size_t)tok * D + col * EPL) * sizeof(T));
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) d = fmaf(qf[g][e], Elem<T>::get(kv, e), d);
#pragma unroll
                for (int o = 1; o < LPR; o <<= 1) d += __shfl_xor(d, o);
                s[g][it] = (tb + tok < t1) ? d * a.scale_log2 : -INFINITY;
            }
        }
        // online softmax update
        float p[G][NIT];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mx = s[g][0];
#pragma unroll
            for (int it = 1; it < NIT; ++it) mx = fmaxf(mx, s[g][it]);
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            const float mn = fmaxf(m[g], mx);          // finite: the block has a visible token
            const float alpha = exp2f(m[g] - mn);      // exp2(-inf) = 0 on the first block
            float ps = 0.f;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                p[g][it] = exp2f(s[g][it] - mn);
                ps += p[g][it];
            }
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) ps += __shfl_xor(ps, o);
            l[g] = l[g] * alpha + ps;
            m[g] = mn;
#pragma unroll
            for (int i = 0; i < DPL; ++i) acc[g][i] *= alpha;
        }
        // acc[g][dim] += sum_t p[g][t] * V^T[dim][t]
        const char* vpage = page + (size_t)kBlock * D * sizeof(T);
#pragma unroll
        for (int i = 0; i < DPL; ++i) {
            const int dim = lane + 64 * i;
            float vrow[kBlock];
#pragma unroll
            for (int c = 0; c < VLD; ++c) {
                uint4 vv = load_stream16(vpage + ((size_t)dim * kBlock + c * EPL) * sizeof(T));
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    const int t = c * EPL + e;
                    vrow[t] = (tb + t < t1) ? Elem<T>::get(vv, e) : 0.f;   // unused slots may hold NaN
                }
            }
#pragma unroll
            for (int t = 0; t < kBlock; ++t) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float pt = __shfl(p[g][t / TPL], (t % TPL) * LPR);
                    acc[g][i] = fmaf(pt, vrow[t], acc[g][i]);
                }
            }
        }
    }
    // per-wave results to LDS
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (lane == 0) { sm_m[wave * G + g] = m[g]; sm_l[wave * G + g] = l[g]; }
#pragma unroll
        for (int i = 0; i < DPL; ++i) sm_acc[(wave * G + g) * D + lane + 64 * i] = acc[g][i];
    }
    __syncthreads();
    finish_item<QT, D, NW>(a, it4.w, part, kvh, seq, nparts, G, sm_m, sm_l, sm_acc);
}

// ---------------------------------------------------------------------------------------------
// 2b. MFMA partial kernel: bf16, head_dim 128, blocks of 16 or 64 tokens, G <= 16.
//
// Each wave walks PAIRS of 16-token page tiles (32 tokens).  With lane = 16 * j + n:
//   QK^T  S^T[token][head] = K[token][:] . Q[head][:]   as 2 tiles x 4 MFMA 16x16x32
//         A = K rows (lane n picks the tile row's token, j picks the 16-byte chunk 4*kk + j of
//         the row), B = Q (lane n = head, same chunk).  Tile rows are mapped to tokens so that
//         after both tiles lane (n, j) holds the scores of head n for the 8 consecutive
//         pair-local tokens 8j .. 8j+7.
//   PV    O^T[dim][head] += V^T[dim][token] P^T[token][head]   as 8 MFMA 16x16x32 (one per 16 dims)
//         A = V^T rows straight from the page (lane n = dim inside the slice, j = the 8 tokens
//         8j..8j+7: one 16-byte load, since V is stored [dim][token]), B = P in registers.
// The softmax state (m, l) of head n lives in lane column n; rescaling O^T needs no shuffles.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

union Frag {
    uint4 u;
    bf16x8 v;
};

struct PairLoads {
    uint4 k[2][4];   // [tile][kk]
    uint4 v[8];      // [dim slice]
};

// a.tile_shift = log2 of the 16-token tiles per KV block: tile i of a request is tile i % 2^shift of
// its block i >> shift.
template <int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2))) void decode_partial_mfma(const DecodeArgs a) {
    constexpr int D = 128;
    constexpr int GMAX = 16;
    __shared__ float sm_m[NW * GMAX], sm_l[NW * GMAX];
    __shared__ float sm_acc[NW * GMAX * D];   // G <= 16 is enforced on the host

    // Workgroups are handed to the 8 XCDs round-robin.  The KV heads of one work item read the same
    // blocks (one page each), so they are given consecutive slots of ONE XCD: they then run side by
    // side behind one L2 and one set of address translations (xcd_map; otherwise item-major order).
    int item, kvh;
    if (a.xcd_map) {
        const int x = blockIdx.x & 7, slot = blockIdx.x >> 3;
        kvh = slot % a.Hkv;
        item = (slot / a.Hkv) * 8 + x;
    } else {
        item = blockIdx.x / a.Hkv;
        kvh = blockIdx.x % a.Hkv;
    }
    const PlanHeader hdr = load_plan_header(a);        // both loads go out together
    const int n_items = hdr.n_items;
    const int4 it4 = a.items[item < a.max_items ? item : a.max_items - 1];   // the length rides along: one dependent load less
    if (hdr.tag != a.plan_tag || it4.z > (long long)a.max_blocks * a.B) return;   // no plan of this batch, or not of this table
    if (item >= n_items || it4.w >= a.max_items) return;   // (a record slot beyond the workspace: the caller's bound was too small)
    const int seq = it4.x, part = it4.y;
    const int G = a.G;
    const int L = it4.z;
    const int nparts = (L + a.part_tokens - 1) / a.part_tokens;
    const int t0 = part * a.part_tokens;
    const int t1 = min(L, t0 + a.part_tokens);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, j = lane >> 4;

    // B operand of QK^T: Q[head n][chunk 4*kk + j], zero rows for the padding heads
    Frag qf[4];
    {
        const char* qrow = (const char*)a.q + (((size_t)seq * a.Hkv + kvh) * G + (n < G ? n : 0)) * D * 2;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            uint4 v = *(const uint4*)(qrow + (4 * kk + j) * 16);
            if (n >= G) v = make_uint4(0, 0, 0, 0);
            qf[kk].u = v;
        }
    }
    f32x4 o[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) o[s] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    const int32_t* trow = a.table + (size_t)seq * a.max_blocks;
    const int nblk = (t1 + kBlock - 1) / kBlock;       // blocks of the request this item may touch
    // tile row n -> token: rows 4jj + r; block jj / 2, slot 8 * (jj % 2) + r (+4 for tile 1)
    const int krow_blk = n >> 3;                       // which block of the pair (0/1)
    const int krow_slot = ((n >> 2) & 1) * 8 + (n & 3);
    const unsigned k_off = (unsigned)krow_slot * (D * 2) + j * 16;      // + kk * 64, + 4 rows for tile 1
    const int v_blk = j >> 1;
    const unsigned v_off = kBlock * D * 2 + (unsigned)n * (kBlock * 2) + (j & 1) * 16;  // + slice * 16 rows

    const int pair0 = t0 / 32 + wave;
    const int pair_end = (t1 + 31) / 32;

    // Page addresses of this wave's pairs, 32 pairs per register pair: lane 2k + b = block b of the
    // wave's k-th pair of the current batch.  One coalesced table gather and one walk over the range
    // table in the vector lanes, instead of dependent scalar loads in front of every pair's loads.
    auto load_pages = [&](int first_pair) -> unsigned long long {
        const int pr_l = first_pair + (lane >> 1) * NW;
        int b = 2 * pr_l + (lane & 1);
        if (b >= nblk) b = (2 * pr_l < nblk) ? 2 * pr_l : nblk - 1;   // odd tail / beyond the partition
        const int id = min(max(trow[b >> a.tile_shift], 0), a.last_block);
        int first = a.rt.first[0];
        unsigned long long base = (unsigned long long)a.rt.base[0];
        for (int r = 1; r < a.rt.n; ++r) {
            const bool in = id >= a.rt.first[r];
            first = in ? a.rt.first[r] : first;
            base = in ? (unsigned long long)a.rt.base[r] : base;
        }
        return base + (unsigned long long)(id - first) * a.block_bytes + (unsigned long long)kvh * a.page_bytes +
               (unsigned)(b & ((1 << a.tile_shift) - 1)) * (2 * kBlock * D * 2);
    };
    unsigned long long pages = load_pages(pair0);
    int pages_first = pair0;

    auto issue = [&](int pr, PairLoads& ld) {
        int k = (pr - pages_first) / NW;
        if (k >= 32) {
            pages = load_pages(pr);
            pages_first = pr;
            k = 0;
        }
        const unsigned aLo = __builtin_amdgcn_readlane((unsigned)pages, 2 * k);
        const unsigned aHi = __builtin_amdgcn_readlane((unsigned)(pages >> 32), 2 * k);
        const unsigned bLo = __builtin_amdgcn_readlane((unsigned)pages, 2 * k + 1);
        const unsigned bHi = __builtin_amdgcn_readlane((unsigned)(pages >> 32), 2 * k + 1);
        const char* pA = (const char*)(((unsigned long long)aHi << 32) | aLo);
        const char* pB = (const char*)(((unsigned long long)bHi << 32) | bLo);
        const char* kp = (krow_blk ? pB : pA) + k_off;
        const char* vp = (v_blk ? pB : pA) + v_off;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            ld.k[0][kk] = load_stream16(kp + kk * 64);
            ld.k[1][kk] = load_stream16(kp + kk * 64 + 4 * D * 2);
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) ld.v[s] = load_stream16(vp + s * (16 * kBlock * 2));
    };

    auto compute = [&](int pr, PairLoads& ld) {
        f32x4 s0 = (f32x4){0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            Frag k0, k1;
            k0.u = ld.k[0][kk];
            k1.u = ld.k[1][kk];
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0.v, qf[kk].v, s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1.v, qf[kk].v, s1, 0, 0, 0);
        }
        // lane (n, j): scores of head n for tokens tbase + e, e = 0..7
        const int tbase = pr * 32 + 8 * j;
        float sc[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) { sc[e] = s0[e] * a.scale_log2; sc[4 + e] = s1[e] * a.scale_log2; }
        const bool tail = (pr * 32 + 32 > t1);
        if (tail) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tbase + e >= t1) sc[e] = -INFINITY;
        }
        float mx = sc[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sc[e]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mn = fmaxf(m, mx);                 // finite: the pair has a visible token
        const float alpha = __builtin_amdgcn_exp2f(m - mn);
        float ps = 0.f;
        Frag pf;
        unsigned short pb[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float p = __builtin_amdgcn_exp2f(sc[e] - mn);
            ps += p;
            pb[e] = f32_to_bf16_rne(p);
        }
        pf.u = make_uint4(pb[0] | ((unsigned)pb[1] << 16), pb[2] | ((unsigned)pb[3] << 16),
                          pb[4] | ((unsigned)pb[5] << 16), pb[6] | ((unsigned)pb[7] << 16));
        l = l * alpha + ps;
        m = mn;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int s = 0; s < 8; ++s) o[s] *= alpha;
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            Frag vf;
            vf.u = ld.v[s];
            if (tail) {   // slots past the context may hold anything: zero them (0 * NaN = NaN)
                unsigned w[4] = {vf.u.x, vf.u.y, vf.u.z, vf.u.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (tbase + e >= t1) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                vf.u = make_uint4(w[0], w[1], w[2], w[3]);
            }
            o[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf.v, o[s], 0, 0, 0);
        }
    };

    // q must have landed before the loop: otherwise the wait for it is placed inside the loop, where
    // it would also wait for the page loads that were just issued for the next pair
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) asm volatile("" : "+v"(qf[kk].v));

    // two register buffers used alternately, so the loads of the next pair stay in flight while the
    // current pair is computed (no register copies, hence no wait on the younger loads)
    PairLoads bufA, bufB;
    int pr = pair0;
    if (pr < pair_end) {
        issue(pr, bufA);
        // The last pair is computed on a path of its own, so that the steady-state path always has
        // the next pair's 16 loads behind the ones it waits for.
        for (;;) {
            const int pr1 = pr + NW;
            if (pr1 >= pair_end) { compute(pr, bufA); break; }
            issue(pr1, bufB);
            compute(pr, bufA);
            const int pr2 = pr1 + NW;
            if (pr2 >= pair_end) { compute(pr1, bufB); break; }
            issue(pr2, bufA);
            compute(pr1, bufB);
            pr = pr2;
        }
    }


    // l: sum over the 4 token groups j of this head
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (n < G) {
        if (j == 0) { sm_m[wave * G + n] = m; sm_l[wave * G + n] = l; }
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i) sm_acc[(wave * G + n) * D + s * 16 + 4 * j + i] = o[s][i];
    }
    __syncthreads();
    finish_item<bf16_t, D, NW>(a, it4.w, part, kvh, seq, nparts, G, sm_m, sm_l, sm_acc);
}

// ---------------------------------------------------------------------------------------------
// 2c. MFMA partial kernel for FP8 (E4M3) pages: head_dim 128, q and out bf16, G <= 16.
//
// Half the bytes per token, so a wave walks QUADS of 16-token page tiles (64 tokens): the same sixteen
// 16-byte loads per lane and step as the bf16 kernel's pair, each now holding sixteen elements, i.e.
// two MFMA operands after conversion to bf16 (exact: every E4M3 value is a bf16 value).  The matrix
// instructions stay the bf16 ones -- the query is bf16, and there is no MFMA that multiplies bf16 by
// fp8.  With lane = 16 j + n:
//   QK^T  four row sets a = 0..3 of S^T[token][head], 4 MFMA 16x16x32 each.  Row r of set a is token
//         (r & 3) + 4a of tile r >> 2, so lane (n, j) loads K rows of tile n >> 2: chunk c = 0, 1 is
//         bytes 64c + 16j .. + 16 of the row = dims 64c + 16j .. + 16, its low half the operand of
//         k-step 2c and its high half that of k-step 2c + 1 (Q is loaded in the same order of dims).
//         After the four sets lane (n, j) holds the scores of head n for all 16 tokens of tile j.
//   PV    O^T[dim][head] += V^T[dim][token] P^T[token][head], two MFMA per 16 dims: k-slot (j, e) of
//         half h is token 8h + e of tile j.  A = one 16-byte V^T row of tile j (16 tokens of one dim):
//         low half for h = 0, high half for h = 1; B = P of those tokens, already in the lane.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

struct QuadK {
    uint4 k[4][2];   // K rows of a quad: [row set][chunk]
};

// sixteen E4M3 codes -> two operands of eight bf16 each (codes 0..7, codes 8..15)
__device__ __forceinline__ void fp8x16_to_bf16(const uint4& x, Frag& lo, Frag& hi) {
    union { bf16x2_t h; unsigned u; } c[8];
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

template <int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2))) void decode_partial_mfma_fp8(const DecodeArgs a) {
    constexpr int D = 128;
    constexpr int GMAX = 16;
    constexpr int kTileBytes = 2 * kBlock * D;         // K [16][128] then V^T [128][16], one byte each
    __shared__ float sm_m[NW * GMAX], sm_l[NW * GMAX];
    __shared__ float sm_acc[NW * GMAX * D];

    int item, kvh;
    if (a.xcd_map) {
        const int x = blockIdx.x & 7, slot = blockIdx.x >> 3;
        kvh = slot % a.Hkv;
        item = (slot / a.Hkv) * 8 + x;
    } else {
        item = blockIdx.x / a.Hkv;
        kvh = blockIdx.x % a.Hkv;
    }
    const PlanHeader hdr = load_plan_header(a);
    const int n_items = hdr.n_items;
    const int4 it4 = a.items[item < a.max_items ? item : a.max_items - 1];
    if (hdr.tag != a.plan_tag || it4.z > (long long)a.max_blocks * a.B) return;   // no plan of this batch, or not of this table
    if (item >= n_items || it4.w >= a.max_items) return;
    const int seq = it4.x, part = it4.y;
    const int G = a.G;
    const int L = it4.z;
    const int nparts = (L + a.part_tokens - 1) / a.part_tokens;
    const int t0 = part * a.part_tokens;
    const int t1 = min(L, t0 + a.part_tokens);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, j = lane >> 4;

    // B operand of QK^T for k-step kk: Q[head n][dims 64 (kk / 2) + 16 j + 8 (kk % 2) .. + 8]
    Frag qf[4];
    {
        const char* qrow = (const char*)a.q + (((size_t)seq * a.Hkv + kvh) * G + (n < G ? n : 0)) * D * 2;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            uint4 v = *(const uint4*)(qrow + 128 * (kk >> 1) + 32 * j + 16 * (kk & 1));
            if (n >= G) v = make_uint4(0, 0, 0, 0);
            qf[kk].u = v;
        }
    }
    f32x4 o[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) o[s] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    const int32_t* trow = a.table + (size_t)seq * a.max_blocks;
    const int ntile = (t1 + kBlock - 1) / kBlock;      // page tiles of the request this item may touch
    const int tile0 = t0 / kBlock;                     // first page tile of the partition
    const int ktile = n >> 2;                          // tile of the quad this lane's K rows come from
    const unsigned k_off = (unsigned)(n & 3) * D + 16 * j;          // + 4 a rows, + 64 c
    const unsigned v_off = kBlock * D + (unsigned)n * kBlock;       // + 16 s rows of V^T

    const int quad_end = (ntile - tile0 + 3) / 4;      // quads of the partition

    // Page-tile addresses of this wave's quads, 16 quads per register pair: lane 4k + b = tile b of the
    // wave's k-th quad of the current batch.
    auto load_pages = [&](int first_quad) -> unsigned long long {
        int t = tile0 + 4 * (first_quad + (lane >> 2) * NW) + (lane & 3);
        if (t >= ntile) t = ntile - 1;                 // beyond the partition: any valid tile
        const int id = min(max(trow[t >> a.tile_shift], 0), a.last_block);
        int first = a.rt.first[0];
        unsigned long long base = (unsigned long long)a.rt.base[0];
        for (int r = 1; r < a.rt.n; ++r) {
            const bool in = id >= a.rt.first[r];
            first = in ? a.rt.first[r] : first;
            base = in ? (unsigned long long)a.rt.base[r] : base;
        }
        return base + (unsigned long long)(id - first) * a.block_bytes + (unsigned long long)kvh * a.page_bytes +
               (unsigned)(t & ((1 << a.tile_shift) - 1)) * kTileBytes;
    };
    unsigned long long pages = load_pages(wave);
    int pages_first = wave;

    // K of the next quad is requested before the current quad is computed (two K buffers used
    // alternately); V^T has ONE buffer, refilled slice by slice with the next quad's rows as soon as
    // the current quad's PV has read a slice -- those loads then stay in flight through the next
    // quad's QK^T and softmax.  (Two full buffers, as in the bf16 kernel, do not fit next to the
    // operands being converted.)
    uint4 vbuf[8];
    // requests the K rows of quad q; returns where this lane's V^T rows of that quad start
    auto issue_k = [&](int q, QuadK& ld) -> const char* {
        int k = (q - pages_first) / NW;
        if (k >= 16) {
            pages = load_pages(q);
            pages_first = q;
            k = 0;
        }
        unsigned long long pt[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const unsigned lo = __builtin_amdgcn_readlane((unsigned)pages, 4 * k + b);
            const unsigned hi = __builtin_amdgcn_readlane((unsigned)(pages >> 32), 4 * k + b);
            pt[b] = ((unsigned long long)hi << 32) | lo;
        }
        const unsigned long long kpage = ktile == 0 ? pt[0] : ktile == 1 ? pt[1] : ktile == 2 ? pt[2] : pt[3];
        const unsigned long long vpage = j == 0 ? pt[0] : j == 1 ? pt[1] : j == 2 ? pt[2] : pt[3];
        const char* kp = (const char*)kpage + k_off;
#pragma unroll
        for (int ra = 0; ra < 4; ++ra) {
            ld.k[ra][0] = load_stream16(kp + ra * 4 * D);
            ld.k[ra][1] = load_stream16(kp + ra * 4 * D + 64);
        }
        return (const char*)vpage + v_off;
    };

    // all of the wave's work on quad q; `refill`: vnext points at the V^T rows of the wave's next quad
    auto compute = [&](int q, QuadK& ld, auto refill, const char* vnext) {
        constexpr bool REFILL = decltype(refill)::value;
        f32x4 sc4[4];
#pragma unroll
        for (int ra = 0; ra < 4; ++ra) {
            f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                Frag k_lo, k_hi;
                fp8x16_to_bf16(ld.k[ra][c], k_lo, k_hi);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_lo.v, qf[2 * c].v, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_hi.v, qf[2 * c + 1].v, acc, 0, 0, 0);
            }
            sc4[ra] = acc;
        }
        // lane (n, j): scores of head n for tokens tbase + 4 ra + i of the request
        const int tbase = (tile0 + 4 * q + j) * kBlock;
        float sc[16];
#pragma unroll
        for (int ra = 0; ra < 4; ++ra)
#pragma unroll
            for (int i = 0; i < 4; ++i) sc[4 * ra + i] = sc4[ra][i] * a.scale_log2;
        const bool tail = (tile0 + 4 * q + 4) * kBlock > t1;
        if (tail) {
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (tbase + e >= t1) sc[e] = -INFINITY;
        }
        float mx = sc[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sc[e]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mn = fmaxf(m, mx);                 // finite: the quad has a visible token
        const float alpha = __builtin_amdgcn_exp2f(m - mn);
        float ps = 0.f;
        Frag pf[2];
        unsigned short pb[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float p = __builtin_amdgcn_exp2f(sc[e] - mn);
            ps += p;
            pb[e] = f32_to_bf16_rne(p);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
            pf[h].u = make_uint4(pb[8 * h + 0] | ((unsigned)pb[8 * h + 1] << 16), pb[8 * h + 2] | ((unsigned)pb[8 * h + 3] << 16),
                                 pb[8 * h + 4] | ((unsigned)pb[8 * h + 5] << 16), pb[8 * h + 6] | ((unsigned)pb[8 * h + 7] << 16));
        l = l * alpha + ps;
        m = mn;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int s = 0; s < 8; ++s) o[s] *= alpha;
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            Frag vh[2];
            fp8x16_to_bf16(vbuf[s], vh[0], vh[1]);
            if (REFILL) vbuf[s] = load_stream16(vnext + s * (16 * kBlock));
            if (tail) {   // slots past the context may hold anything: zero them (0 * NaN = NaN)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    unsigned w[4] = {vh[h].u.x, vh[h].u.y, vh[h].u.z, vh[h].u.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (tbase + 8 * h + e >= t1) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                    vh[h].u = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            o[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh[0].v, pf[0].v, o[s], 0, 0, 0);
            o[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh[1].v, pf[1].v, o[s], 0, 0, 0);
        }
    };

#pragma unroll
    for (int kk = 0; kk < 4; ++kk) asm volatile("" : "+v"(qf[kk].v));

    using Yes = std::integral_constant<bool, true>;
    using No = std::integral_constant<bool, false>;
    QuadK kA, kB;
    int q = wave;
    if (q < quad_end) {
        const char* v0 = issue_k(q, kA);
#pragma unroll
        for (int s = 0; s < 8; ++s) vbuf[s] = load_stream16(v0 + s * (16 * kBlock));
        // the last quad is computed on a path of its own, so that the steady-state path always has the
        // next quad's loads behind the ones it waits for
        for (;;) {
            const int q1 = q + NW;
            if (q1 >= quad_end) { compute(q, kA, No{}, nullptr); break; }
            const char* v1 = issue_k(q1, kB);
            compute(q, kA, Yes{}, v1);
            const int q2 = q1 + NW;
            if (q2 >= quad_end) { compute(q1, kB, No{}, nullptr); break; }
            const char* v2 = issue_k(q2, kA);
            compute(q1, kB, Yes{}, v2);
            q = q2;
        }
    }

    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (n < G) {
        if (j == 0) { sm_m[wave * G + n] = m; sm_l[wave * G + n] = l; }
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i) sm_acc[(wave * G + n) * D + s * 16 + 4 * j + i] = o[s][i];
    }
    __syncthreads();
    finish_item<bf16_t, D, NW>(a, it4.w, part, kvh, seq, nparts, G, sm_m, sm_l, sm_acc);
}

// ---------------------------------------------------------------------------------------------
// 3. merge as a launch of its own (large batches): workgroups per (request, kv head); only requests
//    with more than one partition have work
// ---------------------------------------------------------------------------------------------
constexpr int kMergeSlices = 4;      // workgroups per (request, kv head): the chain of dependent loads per thread is short
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_merge_kernel(const DecodeArgs a) {
    const int slice = blockIdx.x % kMergeSlices;
    const int seq = blockIdx.x / kMergeSlices / a.Hkv, kvh = blockIdx.x / kMergeSlices % a.Hkv;
    if (load_plan_header(a).tag != a.plan_tag) return;
    const int L = a.ctx_len[seq];
    if (L > (long long)a.max_blocks * a.B) return;      // left out by the partial kernel: no records to merge
    const int nparts = (L + a.part_tokens - 1) / a.part_tokens;
    if (nparts <= 1) return;
    const int first = a.seq_first[seq];
    if (first + nparts > a.max_items) return;   // the caller's bound on sum(ctx_len) was too small
    merge_records<T, D, false>(a, first, nparts, kvh, seq, a.G, slice * 256 + threadIdx.x, kMergeSlices * 256);
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
constexpr int kPartChoices[] = {256, 512, 1024, 2048, 4096, 8192};
constexpr int kNumPartChoices = 6;
constexpr int64_t kFoldMaxTokens = 2000000;   // context tokens up to which the merge is folded into the partial kernel
constexpr int kPartDivisor = 1024;    // aim at >= this many (partition, kv head) workgroups

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// What identifies the plan a call expects to find in its workspace (never 0).
int plan_tag_of(int S, int P, int max_items, int Hkv, int G) {
    uint32_t h = 0x9e3779b9u;
    for (uint32_t v : {(uint32_t)S, (uint32_t)P, (uint32_t)max_items, (uint32_t)Hkv, (uint32_t)G}) {
        h ^= v + 0x9e3779b9u + (h << 6) + (h >> 2);
    }
    return (int)(h | 1u);
}

int64_t default_bound(const kun_kv_pool* p, int S, int64_t ub) {
    const int64_t cap = (int64_t)p->ranges.first[p->ranges.n] * p->B;
    if (ub <= 0 || ub > cap) ub = cap;
    return ub;
}

// Partition size: the largest choice that still leaves about a thousand workgroups (256 CUs, two
// resident workgroups each, and a work list that starts the long partitions first); measured best
// on the 8B/70B-shaped batches.
int choose_part_tokens(const kun_kv_pool* p, int64_t ub) {
    if (kun_options().decode_part > 0) return kun_options().decode_part;
    const int64_t per = ub * p->Hkv / kPartDivisor;
    int P = kPartChoices[0];
    for (int i = 0; i < kNumPartChoices; ++i)
        if (per >= kPartChoices[i]) P = kPartChoices[i];
    return P;
}

struct DecodeLayout {
    size_t off_first, off_arrived, off_items, off_ml, off_acc, total;
    int max_items;
};

DecodeLayout layout_for(const kun_kv_pool* p, int S, int Hq, int64_t ub, int P) {
    DecodeLayout lay;
    const int G = Hq / p->Hkv;
    int64_t mi = ub / P + S;
    lay.max_items = (int)(mi > INT32_MAX / 2 ? INT32_MAX / 2 : mi);
    size_t o = 256;
    lay.off_first = o; o += align256(sizeof(int32_t) * ((size_t)S + 1));
    lay.off_arrived = o; o += align256(sizeof(int32_t) * (size_t)S * p->Hkv);
    lay.off_items = o; o += align256(sizeof(int4) * (size_t)lay.max_items);
    lay.off_ml = o;    o += align256(sizeof(float) * 2 * (size_t)lay.max_items * p->Hkv * G);
    lay.off_acc = o;   o += align256(sizeof(float) * (size_t)lay.max_items * p->Hkv * G * p->d);
    lay.total = o;
    return lay;
}

bool decode_shape_ok(const kun_kv_pool* p, int S, int Hq) {
    if (!p || S < 0 || Hq <= 0 || Hq % p->Hkv != 0) return false;
    return true;
}

template <typename T, int D>
int launch_generic(const DecodeArgs& a, dim3 grid, hipStream_t st) {
    switch (a.G) {
        case 1: hipLaunchKernelGGL((decode_partial_generic<T, D, 1>), grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL((decode_partial_generic<T, D, 2>), grid, dim3(256), 0, st, a); break;
        case 3: hipLaunchKernelGGL((decode_partial_generic<T, D, 3>), grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL((decode_partial_generic<T, D, 4>), grid, dim3(256), 0, st, a); break;
        case 5: hipLaunchKernelGGL((decode_partial_generic<T, D, 5>), grid, dim3(256), 0, st, a); break;
        case 6: hipLaunchKernelGGL((decode_partial_generic<T, D, 6>), grid, dim3(256), 0, st, a); break;
        case 7: hipLaunchKernelGGL((decode_partial_generic<T, D, 7>), grid, dim3(256), 0, st, a); break;
        case 8: hipLaunchKernelGGL((decode_partial_generic<T, D, 8>), grid, dim3(256), 0, st, a); break;
        default: return KUN_ERR_UNSUPPORTED;
    }
    return KUN_OK;
}

int launch_generic_any(const kun_kv_pool* p, const DecodeArgs& a, dim3 grid, hipStream_t st) {
    if (p->dtype == KUN_BF16)
        return p->d == 128 ? launch_generic<bf16_t, 128>(a, grid, st) : launch_generic<bf16_t, 64>(a, grid, st);
    if (p->dtype == KUN_FP8_E4M3)
        return p->d == 128 ? launch_generic<fp8_t, 128>(a, grid, st) : launch_generic<fp8_t, 64>(a, grid, st);
    return p->d == 128 ? launch_generic<float, 128>(a, grid, st) : launch_generic<float, 64>(a, grid, st);
}

// every row is its own request with one partition: item t = (t, 0)
__global__ __launch_bounds__(256) void rows_plan_kernel(int T, int32_t* __restrict__ n_items,
                                                        int32_t* __restrict__ seq_first, int4* __restrict__ items,
                                                        const int32_t* __restrict__ ctx_len, int tag) {
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t <= T; t += gridDim.x * blockDim.x) {
        seq_first[t] = t;
        if (t < T) items[t] = make_int4(t, 0, ctx_len[t], 0);
        if (t == 0) { n_items[0] = T; n_items[1] = tag; }
    }
}

}  // namespace

size_t kun_attend_rows_workspace_bytes(int T) {
    return 256 + align256(sizeof(int32_t) * ((size_t)T + 1)) + align256(sizeof(int4) * (size_t)T);
}

int kun_attend_rows_generic(const kun_kv_pool* p, const void* q, void* out, const int32_t* table, int max_blocks,
                            const int32_t* ctx_len, const int32_t* row_of_seq, int T, int Hq, float scale,
                            void* workspace, hipStream_t st) {
    char* ws = (char*)workspace;
    DecodeArgs a;
    a.rt = p->ranges;
    a.q = q;
    a.out = out;
    a.table = table;
    a.ctx_len = ctx_len;
    a.row_of_seq = row_of_seq;
    a.n_items = (int32_t*)ws;
    a.seq_first = (int32_t*)(ws + 256);
    a.items = (int4*)(ws + 256 + align256(sizeof(int32_t) * ((size_t)T + 1)));
    a.arrived = nullptr;          // one partition per row: outputs are written directly
    a.part_ml = nullptr;
    a.part_acc = nullptr;
    a.max_blocks = max_blocks;
    a.S = T;
    a.Hkv = p->Hkv;
    a.G = Hq / p->Hkv;
    a.B = p->B;
    a.last_block = p->ranges.first[p->ranges.n] - 1;
    a.tile_shift = p->B == 128 ? 3 : p->B == 64 ? 2 : p->B == 32 ? 1 : 0;
    a.part_tokens = 1 << 30;
    a.max_items = T;
    a.scale_log2 = scale * kLog2e;
    a.block_bytes = (unsigned)p->block_bytes;
    a.page_bytes = (unsigned)p->page_bytes;
    a.xcd_map = 0;
    a.fold = 0;
    a.plan_tag = plan_tag_of(T, 0, T, p->Hkv, a.G);
    const int nb = (T + 256) / 256;
    hipLaunchKernelGGL(rows_plan_kernel, dim3((unsigned)(nb < 1024 ? nb : 1024)), dim3(256), 0, st, T, a.n_items,
                       a.seq_first, a.items, ctx_len, a.plan_tag);
    KUN_HIP_CHECK_LAUNCH();
    const dim3 grid((unsigned)((size_t)T * p->Hkv));
    const int rc = launch_generic_any(p, a, grid, st);
    if (rc != KUN_OK) return rc;
    KUN_HIP_CHECK_LAUNCH();
    return KUN_OK;
}

namespace {
enum DecodeSteps { kPlanAndRun = 0, kPlanOnly = 1, kRunOnly = 2 };
int decode_enqueue(kun_kv_pool* p, const void* q, void* out, const int32_t* block_table, int max_blocks,
                   const int32_t* ctx_len, int S, int Hq, float scale, int64_t ub, void* workspace,
                   size_t workspace_bytes, void* stream, DecodeSteps steps = kPlanAndRun);
}

extern "C" {

size_t kun_decode_workspace_bytes(const kun_kv_pool* p, int S, int Hq, int64_t ub) {
    if (!decode_shape_ok(p, S, Hq)) return 0;
    ub = default_bound(p, S, ub);
    // The partition size steps up with the bound; size for the worst case at or below `ub`.
    size_t need = layout_for(p, S, Hq, ub, choose_part_tokens(p, ub)).total;
    for (int i = 1; i < kNumPartChoices; ++i) {
        const int64_t edge = ((int64_t)kPartChoices[i] * kPartDivisor + p->Hkv - 1) / p->Hkv - 1;   // last bound using choice i-1
        if (edge < ub && edge > 0) {
            size_t n2 = layout_for(p, S, Hq, edge, choose_part_tokens(p, edge)).total;
            if (n2 > need) need = n2;
        }
    }
    return need;
}

int kun_paged_decode(kun_kv_pool* p, const void* q, void* out, const int32_t* block_table,
                     int max_blocks, const int32_t* ctx_len, int S, int Hq, float scale,
                     int64_t ub, void* workspace, size_t workspace_bytes, void* stream) {
    return decode_enqueue(p, q, out, block_table, max_blocks, ctx_len, S, Hq, scale, ub, workspace, workspace_bytes,
                          stream);
}

int kun_decode_plan(kun_kv_pool* p, const int32_t* ctx_len, int S, int Hq, int64_t ub, void* workspace,
                    size_t workspace_bytes, void* stream) {
    return decode_enqueue(p, nullptr, nullptr, nullptr, 0, ctx_len, S, Hq, 1.0f, ub, workspace, workspace_bytes,
                          stream, kPlanOnly);
}

int kun_paged_decode_planned(kun_kv_pool* p, const void* q, void* out, const int32_t* block_table,
                             int max_blocks, const int32_t* ctx_len, int S, int Hq, float scale,
                             int64_t ub, void* workspace, size_t workspace_bytes, void* stream) {
    return decode_enqueue(p, q, out, block_table, max_blocks, ctx_len, S, Hq, scale, ub, workspace, workspace_bytes,
                          stream, kRunOnly);
}

}  // extern "C"

namespace {

int decode_enqueue(kun_kv_pool* p, const void* q, void* out, const int32_t* block_table,
                   int max_blocks, const int32_t* ctx_len, int S, int Hq, float scale,
                   int64_t ub, void* workspace, size_t workspace_bytes, void* stream, DecodeSteps steps) {
    if (!decode_shape_ok(p, S, Hq)) return KUN_ERR_INVALID_ARG;
    if (S == 0) return KUN_OK;
    if (!ctx_len) return KUN_ERR_INVALID_ARG;
    if (steps != kPlanOnly && (!q || !out || !block_table || max_blocks <= 0)) return KUN_ERR_INVALID_ARG;
    const int G = Hq / p->Hkv;
    const bool generic_only = kun_options().decode_generic;
    const bool mfma = (p->dtype == KUN_BF16 || p->dtype == KUN_FP8_E4M3) && p->d == 128 && !generic_only;
    if (G < 1 || (G > 8 && !(G == 16 && mfma))) return KUN_ERR_UNSUPPORTED;   // 16 heads per KV head: the MFMA kernel only
    ub = default_bound(p, S, ub);
    const int P = choose_part_tokens(p, ub);
    const DecodeLayout lay = layout_for(p, S, Hq, ub, P);
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < lay.total)
        return KUN_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;

    DecodeArgs a;
    a.rt = p->ranges;
    a.q = q;
    a.out = out;
    a.table = block_table;
    a.ctx_len = ctx_len;
    a.row_of_seq = nullptr;
    a.n_items = (int32_t*)ws;
    a.seq_first = (int32_t*)(ws + lay.off_first);
    a.items = (int4*)(ws + lay.off_items);
    a.arrived = (int32_t*)(ws + lay.off_arrived);
    a.part_ml = (float*)(ws + lay.off_ml);
    a.part_acc = (float*)(ws + lay.off_acc);
    a.max_blocks = max_blocks;
    a.S = S;
    a.Hkv = p->Hkv;
    a.G = G;
    a.B = p->B;
    a.last_block = p->ranges.first[p->ranges.n] - 1;
    a.tile_shift = p->B == 128 ? 3 : p->B == 64 ? 2 : p->B == 32 ? 1 : 0;
    a.part_tokens = P;
    a.max_items = lay.max_items;
    a.scale_log2 = scale * kLog2e;
    a.block_bytes = (unsigned)p->block_bytes;
    a.page_bytes = (unsigned)p->page_bytes;
    a.xcd_map = 0;
    // Small batches: the merge rides in the partial kernel (one launch and one gap less, worth 2 % of
    // a 0.5 ms call).  Large ones: a launch of its own (there the wait for the arrival count at the end
    // of every workgroup costs more than the launch: 4 % of a 2.6 ms call).
    const int merge_opt = kun_options().decode_merge;
    a.fold = merge_opt == 1 || (merge_opt == 0 && ub <= kFoldMaxTokens);
    a.plan_tag = plan_tag_of(S, P, lay.max_items, p->Hkv, G);

    if (steps != kRunOnly) {
        hipLaunchKernelGGL(decode_plan_kernel, dim3(1), dim3(1024), 0, st, ctx_len, S, P, lay.max_items,
                           a.n_items, a.seq_first, a.items, a.arrived, S * p->Hkv, a.plan_tag);
        KUN_HIP_CHECK_LAUNCH();
    }
    if (steps == kPlanOnly) return KUN_OK;

    dim3 grid((unsigned)((size_t)lay.max_items * p->Hkv));
    int rc = KUN_OK;
    if (mfma) {
        const int nw = kun_options().decode_waves;
        a.xcd_map = !kun_options().decode_flat_map;
        if (a.xcd_map) grid = dim3((unsigned)(((size_t)lay.max_items + 7) / 8 * 8 * p->Hkv));
        if (p->dtype == KUN_FP8_E4M3) {
            if (nw == 1) hipLaunchKernelGGL((decode_partial_mfma_fp8<1>), grid, dim3(64), 0, st, a);
            else if (nw == 2) hipLaunchKernelGGL((decode_partial_mfma_fp8<2>), grid, dim3(128), 0, st, a);
            else hipLaunchKernelGGL((decode_partial_mfma_fp8<4>), grid, dim3(256), 0, st, a);
        } else {
            if (nw == 1) hipLaunchKernelGGL((decode_partial_mfma<1>), grid, dim3(64), 0, st, a);
            else if (nw == 2) hipLaunchKernelGGL((decode_partial_mfma<2>), grid, dim3(128), 0, st, a);
            else hipLaunchKernelGGL((decode_partial_mfma<4>), grid, dim3(256), 0, st, a);
        }
    } else {
        rc = launch_generic_any(p, a, grid, st);
    }
    if (rc != KUN_OK) return rc;
    KUN_HIP_CHECK_LAUNCH();
    if (!a.fold) {
        const dim3 mgrid((unsigned)((size_t)S * p->Hkv * kMergeSlices));
        const bool out_bf16 = p->dtype != KUN_F32;     // outputs of bf16 and of FP8 pools are bf16
        if (out_bf16 && p->d == 128) hipLaunchKernelGGL((decode_merge_kernel<bf16_t, 128>), mgrid, dim3(256), 0, st, a);
        else if (out_bf16) hipLaunchKernelGGL((decode_merge_kernel<bf16_t, 64>), mgrid, dim3(256), 0, st, a);
        else if (p->d == 128) hipLaunchKernelGGL((decode_merge_kernel<float, 128>), mgrid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((decode_merge_kernel<float, 64>), mgrid, dim3(256), 0, st, a);
        KUN_HIP_CHECK_LAUNCH();
    }
    return KUN_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Decode without a caller-provided workspace, for callers that cannot allocate one (code under HIP
// graph capture, tight serving loops, harnesses that forbid allocation): the split-K records live in
// a fixed array in the library's own device image.  Every GPU the library runs on holds its own copy
// of the array, at its own address, until the process ends.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[KUN_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];     // device address of `scratch` on each device, looked up once

// Device address of the current device's copy of `scratch` (the array's name is only a host-side
// stand-in: host code always goes through this pointer).
int static_scratch(void** out) {
    int dev = 0;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { kun_note_hip_error("hipGetDevice", e); return KUN_ERR_HIP; }
    if (dev < 0 || dev >= kMaxDevices) return KUN_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e2 = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (e2 != hipSuccess || !ptr) { kun_note_hip_error("hipGetSymbolAddress", e2); return KUN_ERR_HIP; }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return KUN_OK;
}

}  // namespace

extern "C" int kun_paged_decode_static(kun_kv_pool* p, const void* q, void* out, const int32_t* block_table,
                                       int max_blocks, const int32_t* ctx_len, int S, int Hq, float scale,
                                       int64_t ub, void* stream) {
    if (!decode_shape_ok(p, S, Hq)) return KUN_ERR_INVALID_ARG;
    if (S == 0) return KUN_OK;
    const size_t need = kun_decode_workspace_bytes(p, S, Hq, ub);
    if (need == 0) return KUN_ERR_INVALID_ARG;
    if (need > (size_t)KUN_STATIC_SCRATCH_BYTES) return KUN_ERR_SCRATCH_LIMIT;
    void* ptr = nullptr;
    const int st = static_scratch(&ptr);
    if (st != KUN_OK) return st;
    return decode_enqueue(p, q, out, block_table, max_blocks, ctx_len, S, Hq, scale, ub, ptr,
                          (size_t)KUN_STATIC_SCRATCH_BYTES, stream);
}
