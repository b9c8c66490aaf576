// Stand-alone measurement of what the two rooflines of the paged-attention path can reach on the
// GPU at hand: it is not part of libkun.so and shares nothing with it.
//
//   1. HBM streaming read: 16 GiB read with grid-stride 16-byte loads, and 17 GB read as scattered
//      8 KiB pieces at 64 KiB granularity (the footprint of one KV head's K + V^T page inside a
//      block of the pool) out of a 16 GiB and out of a 150 GiB buffer, each with ordinary and with
//      non-temporal loads.  This is the ceiling of the decode step, which the paper classes as
//      memory-bound (section 2.1).
//   2. MFMA issue rate of v_mfma_f32_32x32x16_bf16 at two waves per SIMD with constant and with
//      random operands (the clock the chip sustains depends on how much the operands toggle).
//   3. The skeleton of a chunked-prefill tile loop (compute-bound per section 2.1): per 64-key
//      tile and wave 16 MFMAs for S^T = K Q^T, the softmax numerators of the 32 x 64 scores against
//      a reference maximum that is checked through the row sums, 16 MFMAs
//      for O^T += V^T P^T, operands read from a 4-stage LDS ring, one barrier per tile, four
//      direct global->LDS loads per lane and tile; every wave does the same work, nothing is
//      masked, the source stays in L2.  Constant and random operands; variants add one cost at a
//      time to the bare MFMA loop (barrier, global->LDS loads, LDS fragment reads, softmax).
//
// Build: python -m paper_2412_18169_amd.build   (writes paper_2412_18169_amd/kun_ceilings)
// Run:   ./paper_2412_18169_amd/kun_ceilings [hbm|mfma|tile|all]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
union Frag {
    uint4 u;
    bf16x8 v;
};

#define CK(x)                                                                         \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                             \
        }                                                                             \
    } while (0)

template <typename F>
static float time_ms(F launch, int reps) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int r = 0; r < reps; ++r) launch();
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms / reps;
}

// ---------------------------------------------------------------- 1. HBM read
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>     // NT: non-temporal loads (data that is read once)
__global__ __launch_bounds__(256) void read_linear(const u32x4* __restrict__ p, size_t n, unsigned* sink) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    unsigned s = 0;
    for (; i + 7 * stride < n; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = NT ? __builtin_nontemporal_load(p + i + u * stride) : p[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u].x ^ v[u].w;
    }
    for (; i < n; i += stride) s += p[i].x;
    if (s == 0x12345678u) sink[0] = s;
}

// The decode kernel's pattern: a workgroup of 4 waves walks `blocks_per_wg` hashed 64 KiB blocks of the
// buffer for one of 8 KV heads; a wave takes two blocks per step and reads the head's 8 KiB page (K +
// V^T) of each with sixteen 16-byte loads per lane.
// XCD: the 8 heads of a group of blocks take consecutive slots of one XCD (workgroups go to the 8
// XCDs round-robin) instead of one slot on each.
template <bool NT, bool XCD>
__global__ __launch_bounds__(256) void read_pages(const u32x4* __restrict__ p, size_t nblocks, int blocks_per_wg,
                                                  unsigned* sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned slot = blockIdx.x >> 3;
    const int head = XCD ? (slot & 7) : (blockIdx.x & 7);
    const size_t group = XCD ? (size_t)(slot >> 3) * 8 + (blockIdx.x & 7) : slot;
    unsigned s = 0;
    const size_t first = group * blocks_per_wg;
    for (int b = wave * 2; b < blocks_per_wg; b += 8) {
        u32x4 v[16];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const size_t blk = ((first + b + h) * 2654435761ull) % nblocks;
            const u32x4* page = p + blk * 4096 + head * 512 + lane;
#pragma unroll
            for (int u = 0; u < 8; ++u) v[8 * h + u] = NT ? __builtin_nontemporal_load(page + u * 64) : page[u * 64];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) s += v[u].x ^ v[u].w;
    }
    if (s == 0x12345678u) sink[0] = s;
}

static void run_hbm(size_t gib) {
    const size_t bytes = gib << 30, n = bytes / 16, nblocks = bytes / 65536;
    u32x4* buf;
    unsigned* sink;
    CK(hipMalloc(&buf, bytes));
    CK(hipMalloc(&sink, 4));
    CK(hipMemset(buf, 1, bytes));
    const size_t lin = bytes < ((size_t)16 << 30) ? bytes : (size_t)16 << 30;      // linear: the first 16 GiB
    const float t0 = time_ms([&] { read_linear<false><<<16384, 256>>>(buf, lin / 16, sink); }, 5);
    const float t1 = time_ms([&] { read_linear<true><<<16384, 256>>>(buf, lin / 16, sink); }, 5);
    std::printf("hbm linear read of 16 GiB, %zu GiB buffer:              %.0f GB/s | non-temporal loads %.0f GB/s\n", gib,
                lin / t0 / 1e6, lin / t1 / 1e6);
    const int bpw = 64;                                    // 64 blocks = 1024 tokens per workgroup
    const size_t wg_groups = 260000 / bpw / 8 * 8;         // about 17 GB, the 70B-shaped decode step
    const double page_bytes = (double)wg_groups * bpw * 8 * 8192;
    const float t2 = time_ms([&] { read_pages<false, false><<<(unsigned)(wg_groups * 8), 256>>>(buf, nblocks, bpw, sink); }, 3);
    const float t3 = time_ms([&] { read_pages<true, false><<<(unsigned)(wg_groups * 8), 256>>>(buf, nblocks, bpw, sink); }, 3);
    const float t4 = time_ms([&] { read_pages<true, true><<<(unsigned)(wg_groups * 8), 256>>>(buf, nblocks, bpw, sink); }, 3);
    std::printf("hbm scattered 8 KiB pages (17 GB of a %zu GiB buffer):  %.0f GB/s | non-temporal loads %.0f GB/s | and the 8 heads"
                " of a block on one XCD %.0f GB/s\n", gib, page_bytes / t2 / 1e6, page_bytes / t3 / 1e6, page_bytes / t4 / 1e6);
    CK(hipFree(buf));
    CK(hipFree(sink));
}

// bf16 bit patterns: constant 1.0, or sign/mantissa/low exponent bits from a linear congruential stream
static std::vector<unsigned> operand_words(size_t nwords, bool random) {
    std::vector<unsigned> h(nwords);
    unsigned x = 99;
    for (size_t i = 0; i < nwords; ++i) {
        unsigned w = 0;
        for (int half = 0; half < 2; ++half) {
            x = x * 1664525u + 1013904223u;
            w |= (0x3d00u + ((x >> 8) & 0x1ff) + ((x >> 31) << 15)) << (16 * half);
        }
        h[i] = random ? w : 0x3f803f80u;
    }
    return h;
}

// ---------------------------------------------------------------- 2. MFMA rate
__global__ __launch_bounds__(512) void mfma_rate(float* out, const uint4* src, int iters) {
    Frag a[8], b[8];
    for (int i = 0; i < 8; ++i) {
        a[i].u = src[(threadIdx.x * 8 + i) & 4095];
        b[i].u = src[(threadIdx.x * 8 + i + 2048) & 4095];
    }
    f32x16 acc[4];
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 16; ++i) acc[k][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j].v, b[(j + k) & 7].v, acc[k], 0, 0, 0);
    }
    float s = 0.f;
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 16; ++i) s += acc[k][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

static void run_mfma(float* out, uint4* src) {
    const int iters = 8000;
    for (int random = 0; random < 2; ++random) {
        const std::vector<unsigned> h = operand_words(4096 * 4, random);
        CK(hipMemcpy(src, h.data(), 4096 * 16, hipMemcpyHostToDevice));
        const float ms = time_ms([&] { mfma_rate<<<256, 512>>>(out, src, iters); }, 3);
        std::printf("mfma 32x32x16 bf16, 2 waves/SIMD, %s operands: %.0f TFLOP/s\n", random ? "random  " : "constant",
                    256.0 * 8 * iters * 32 * 32768.0 / ms / 1e9);
    }
}

// ---------------------------------------------------------------- 3. attention tile loop
// One cost at a time on top of the bare MFMA loop (32 MFMAs per tile and wave, operands in registers):
// LD:   0 = every K / V^T fragment is read from LDS (32 ds_read_b128 per tile and wave), 1 = every
//       fragment read feeds two MFMAs (16 reads; a second Q fragment, a repeated V^T fragment: wrong
//       results, the same number of MFMAs and softmax instructions), 2 = none (fragments read once
//       before the loop).
// SM:   the softmax numerators (fma, exp2, row sums, conversion to bf16) or only the conversion.
// SYNC: 0 = none, 1 = the barrier and the four global->LDS loads per lane and tile, 2 = the barrier
//       only, 3 = the loads (and the wait for the tile loaded three iterations earlier) only.
template <int LD, bool SM, int SYNC>
__global__ __launch_bounds__(512) void tile_loop(float* out, const uint4* gsrc, int iters, float sl2) {
    __shared__ __attribute__((aligned(16))) unsigned char ring[4][32768];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, jh = lane >> 5;
    for (int i = tid; i < 4 * 32768 / 16; i += 512) ((uint4*)&ring[0][0])[i] = gsrc[(i * 7 + blockIdx.x) & 8191];
    __syncthreads();
    Frag q, q2;
    q.u = gsrc[tid * 3 + 5];
    q2.u = gsrc[tid * 5 + 11];
    f32x16 o[4];
    for (int i = 0; i < 16; ++i)
        for (int d = 0; d < 4; ++d) o[d][i] = 0;
    float m = 0.f, l = 0.f;
    // score row r of the 32 x 32 tile holds key krow, so that a lane's 8 scores per PV step are 8
    // consecutive keys = one 16-byte read of a V^T row
    const int krow = 16 * (n >> 4) + 8 * ((n >> 2) & 1) + 4 * ((n >> 3) & 1) + (n & 3);
    const int krow_blk = krow >> 4, krow_in = krow & 15;
    const unsigned k_lane = krow_blk * 4096 + krow_in * 256;
    const unsigned v_lane = 16384 + n * 32 + ((jh ^ ((n >> 3) & 1)) * 16);
    const unsigned ring_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)&ring[0][0];
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    Frag ka[8];
    for (int ks = 0; ks < 8; ++ks) ka[ks].u = *(const uint4*)(&ring[0][0] + k_lane + (((2 * ks + jh) ^ krow_in) * 16));
    // everything loaded so far has landed before the loop: otherwise the compiler puts its waits for
    // these operands inside the loop, where a vmcnt(0) also waits for the tile loads just issued
    asm volatile("" : "+v"(q.v), "+v"(q2.v));
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(ka[ks].v));
    for (int it = 0; it < iters; ++it) {
        if (SYNC) {
            if (SYNC != 2) __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8)
            if (SYNC != 3) __builtin_amdgcn_s_barrier();
            if (SYNC != 2) {
                const unsigned st = ring_addr + ((it + 3) & 3) * 32768 + (wave_u & 3) * 1024;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const char* page = (const char*)(gsrc + ((size_t)((it * 7 + wave_u * 2 + i) & 1023)) * 512);
                    const unsigned dk = st + ((wave_u >> 2) + 2 * i) * 4096;
                    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(page + lane * 16), "s"(dk) : "memory", "m0");
                    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(page + 4096 + lane * 16), "s"(dk + 16384) : "memory", "m0");
                }
            }
        }
        const unsigned char* stage_base = &ring[it & 3][0];
        f32x16 sa, sb;
        for (int i = 0; i < 16; ++i) {
            sa[i] = 0.f;
            sb[i] = 0.f;
        }
        const unsigned char* kbase = stage_base + k_lane;
        Frag kb[8];
        if (LD != 2) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const unsigned off = ((2 * ks + jh) ^ krow_in) * 16;
                ka[ks].u = *(const uint4*)(kbase + off);
                if (LD == 0) kb[ks].u = *(const uint4*)(kbase + 8192 + off);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks].v, q.v, sa, 0, 0, 0);
            if (LD != 0) sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks].v, q2.v, sb, 0, 0, 0);
            else sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[ks].v, q.v, sb, 0, 0, 0);
        }
        const unsigned char* vbase = stage_base + v_lane;
        Frag vf[16];
#pragma unroll
        for (int h = 0; h < 4; ++h)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if (LD == 2) vf[4 * h + d].u = ka[(4 * h + d) & 7].u;
                else if (LD == 1 && h >= 2) vf[4 * h + d].u = vf[4 * (h - 2) + d].u;
                else vf[4 * h + d].u = *(const uint4*)(vbase + h * 4096 + d * 1024);
            }
        __builtin_amdgcn_sched_barrier(0);
        float ps0 = 0, ps1 = 0;
        union {
            bf16x2 h[16];
            uint4 u[4];
        } cv;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            float p0 = sa[i], p1 = sa[i + 1], p2 = sb[i], p3 = sb[i + 1];
            if (SM) {
                p0 = __builtin_amdgcn_exp2f(fmaf(p0, sl2, -m));
                p1 = __builtin_amdgcn_exp2f(fmaf(p1, sl2, -m));
                p2 = __builtin_amdgcn_exp2f(fmaf(p2, sl2, -m));
                p3 = __builtin_amdgcn_exp2f(fmaf(p3, sl2, -m));
                ps0 += p0 + p2;
                ps1 += p1 + p3;
            }
            cv.h[i >> 1] = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
            cv.h[8 + (i >> 1)] = __builtin_convertvector((f32x2){p2, p3}, bf16x2);
        }
        if (SM) {
            const float pt = ps0 + ps1;
            if (__builtin_amdgcn_ballot_w64(!(pt <= 8192.f)) != 0) m += 1.f;  // stale reference maximum (never with these operands)
            l += pt;
        }
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            Frag pb;
            pb.u = cv.u[h];
#pragma unroll
            for (int d = 0; d < 4; ++d) o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[4 * h + d].v, pb.v, o[d], 0, 0, 0);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no load into LDS may outlive the workgroup
    float s = l + m;
    for (int i = 0; i < 16; ++i)
        for (int d = 0; d < 4; ++d) s += o[d][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}


#define KUN_TILE(LD, SM, SYNC) time_ms([&] { tile_loop<LD, SM, SYNC><<<256, 512>>>(out, src, iters, 0.01f); }, 1)
static void run_tile(float* out, uint4* src) {
    const int iters = 4000;
    const double flops = 256.0 * 8 * iters * 32 * 32768.0;
    for (int random = 0; random < 2; ++random) {
        const std::vector<unsigned> h = operand_words(1024 * 8192 / 4, random);
        CK(hipMemcpy(src, h.data(), 1024 * 8192, hipMemcpyHostToDevice));
        // the variants take turns and the best of five rounds counts: the clock drifts by several
        // percent over the first launches of a session
        const int N = 8;
        float best[N];
        for (int i = 0; i < N; ++i) best[i] = 1e9f;
        for (int round = 0; round < 5; ++round) {
            const float t[N] = {KUN_TILE(2, false, 0), KUN_TILE(2, false, 2), KUN_TILE(0, false, 0), KUN_TILE(1, false, 0),
                                KUN_TILE(2, true, 0),  KUN_TILE(0, true, 0),  KUN_TILE(1, true, 1),  KUN_TILE(0, true, 1)};
            for (int i = 0; i < N; ++i) best[i] = t[i] < best[i] ? t[i] : best[i];
        }
        // (the loads are not shown on their own: next to the bare loop they would run at a tile rate,
        // and so at a load rate, that the full loop never reaches)
        const char* names[N] = {"bare MFMA loop", "+ barrier", "+ LDS fragment reads", "+ half of them", "+ softmax",
                                "+ reads and softmax", "all, half of the reads", "all = + barrier and global->LDS loads"};
        std::printf("attention tile loop, %s operands, TFLOP/s:", random ? "random  " : "constant");
        for (int i = 0; i < N; ++i) std::printf(" %s %.0f%s", names[i], flops / best[i] / 1e9, i + 1 < N ? " |" : "\n");
    }
}

int main(int argc, char** argv) {
    const char* what = argc > 1 ? argv[1] : "all";
    const bool all = !std::strcmp(what, "all");
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    std::printf("device: %s (%s), %d CUs\n", prop.name, prop.gcnArchName, prop.multiProcessorCount);
    float* out;
    uint4* src;
    CK(hipMalloc(&out, 256 * 512 * sizeof(float)));
    CK(hipMalloc(&src, 1024 * 8192));
    if (all || !std::strcmp(what, "mfma")) run_mfma(out, src);
    if (all || !std::strcmp(what, "tile")) run_tile(out, src);
    if (all || !std::strcmp(what, "hbm")) {
        run_hbm(16);
        run_hbm(150);     // the size of the largest pool: scattered pages now also miss in the TLBs
    }
    CK(hipFree(out));
    CK(hipFree(src));
    return 0;
}
