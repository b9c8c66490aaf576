// Virtual-memory form of the KVCache region (Section 4.1, "Local instance memory management"): one
// virtual address range is reserved for the largest KVCache the instance may ever hold, physical
// memory is mapped at its tail when the pool grows, and the physical chunks behind dropped
// parameters are remapped there without a copy (and back on restoration, Section 4.4).  Kernels then see ONE contiguous
// range whose size changes; kun_kv_pool_resize_tail tells the pool.
//
// Host code only (HIP virtual memory management API); no kernels.
#include <new>
#include <vector>

#include "kun_internal.h"

struct kun_vmm_region {
    char* base = nullptr;
    size_t reserved = 0, mapped = 0, gran = 0;
    int device = 0;
    struct Chunk {
        hipMemGenericAllocationHandle_t handle;
        size_t bytes;
    };
    std::vector<Chunk> chunks;     // in address order; chunk i starts where chunk i-1 ends
};

namespace {

constexpr size_t kMinGranularity = (size_t)2 << 20;

// true if the call failed (and notes it for kun_last_hip_error)
bool failed(const char* call, hipError_t e) {
    if (e == hipSuccess) return false;
    kun_note_hip_error(call, e);
    return true;
}

hipMemAllocationProp device_prop(int device) {
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device;
    return prop;
}

int map_at_tail(kun_vmm_region* r, hipMemGenericAllocationHandle_t h, size_t bytes) {
    if (r->mapped + bytes > r->reserved) return KUN_ERR_TOO_SMALL;
    char* at = r->base + r->mapped;
    if (failed("hipMemMap", hipMemMap(at, bytes, 0, h, 0))) return KUN_ERR_HIP;
    hipMemAccessDesc acc = {};
    acc.location.type = hipMemLocationTypeDevice;
    acc.location.id = r->device;
    acc.flags = hipMemAccessFlagsProtReadWrite;
    // Access is set for everything mapped so far, not for the new chunk alone: asked for a chunk that
    // is not the first of its reservation, this driver answers "invalid argument" unless all chunks
    // have the same size (measured: a call over [base, end of the new chunk) never failed, for fresh
    // and for remapped allocation handles).
    if (failed("hipMemSetAccess", hipMemSetAccess(r->base, r->mapped + bytes, &acc, 1))) {
        (void)hipMemUnmap(at, bytes);
        return KUN_ERR_HIP;
    }
    r->chunks.push_back({h, bytes});
    r->mapped += bytes;
    return KUN_OK;
}

// number of tail chunks that make up exactly `bytes`; 0 if no whole number of chunks does
size_t tail_chunks(const kun_vmm_region* r, size_t bytes) {
    size_t n = 0, sum = 0;
    while (sum < bytes && n < r->chunks.size()) sum += r->chunks[r->chunks.size() - 1 - n++].bytes;
    return sum == bytes ? n : 0;
}

}  // namespace

extern "C" {

int kun_vmm_region_create(kun_vmm_region** out, size_t reserve_bytes) {
    if (!out) return KUN_ERR_INVALID_ARG;
    *out = nullptr;
    if (reserve_bytes == 0) return KUN_ERR_INVALID_ARG;
    kun_vmm_region* r = new (std::nothrow) kun_vmm_region();
    if (!r) return KUN_ERR_INVALID_ARG;
    if (failed("hipGetDevice", hipGetDevice(&r->device))) { delete r; return KUN_ERR_HIP; }
    const hipMemAllocationProp prop = device_prop(r->device);
    if (failed("hipMemGetAllocationGranularity",
               hipMemGetAllocationGranularity(&r->gran, &prop, hipMemAllocationGranularityRecommended)) ||
        r->gran == 0) {
        delete r;
        return KUN_ERR_HIP;
    }
    // The driver reports 4 KiB here; the region works in units of at least 2 MiB, base included, so
    // that chunks can be mapped with large pages.
    if (r->gran < kMinGranularity) r->gran = kMinGranularity;
    r->reserved = (reserve_bytes + r->gran - 1) / r->gran * r->gran;
    void* va = nullptr;
    if (failed("hipMemAddressReserve", hipMemAddressReserve(&va, r->reserved, r->gran, nullptr, 0))) {
        delete r;
        return KUN_ERR_HIP;
    }
    r->base = (char*)va;
    *out = r;
    return KUN_OK;
}

int kun_vmm_region_info(const kun_vmm_region* r, void** base, size_t* mapped_bytes, size_t* reserved_bytes,
                        size_t* granularity) {
    if (!r) return KUN_ERR_INVALID_ARG;
    if (base) *base = r->base;
    if (mapped_bytes) *mapped_bytes = r->mapped;
    if (reserved_bytes) *reserved_bytes = r->reserved;
    if (granularity) *granularity = r->gran;
    return KUN_OK;
}

int kun_vmm_region_grow(kun_vmm_region* r, size_t bytes) {
    if (!r || bytes == 0) return KUN_ERR_INVALID_ARG;
    if (bytes % r->gran != 0) return KUN_ERR_MISALIGNED;
    if (r->mapped + bytes > r->reserved) return KUN_ERR_TOO_SMALL;
    const hipMemAllocationProp prop = device_prop(r->device);
    hipMemGenericAllocationHandle_t h;
    if (failed("hipMemCreate", hipMemCreate(&h, bytes, &prop, 0))) return KUN_ERR_HIP;
    const int st = map_at_tail(r, h, bytes);
    if (st != KUN_OK) (void)hipMemRelease(h);
    return st;
}

int kun_vmm_region_move_tail(kun_vmm_region* src, kun_vmm_region* dst, size_t bytes) {
    if (!src || !dst || src == dst || bytes == 0) return KUN_ERR_INVALID_ARG;
    const size_t n = tail_chunks(src, bytes);
    if (n == 0) return KUN_ERR_MISALIGNED;
    if (dst->mapped + bytes > dst->reserved) return KUN_ERR_TOO_SMALL;
    if (src->device != dst->device) return KUN_ERR_INVALID_ARG;
    // lowest of the moved chunks first, so their order (and every byte's offset inside the moved
    // span) is the same at the destination
    const size_t first = src->chunks.size() - n;
    size_t off = src->mapped - bytes;
    for (size_t i = first; i < src->chunks.size(); ++i) {
        const kun_vmm_region::Chunk c = src->chunks[i];
        if (failed("hipMemUnmap", hipMemUnmap(src->base + off, c.bytes))) return KUN_ERR_HIP;
        off += c.bytes;
        const int st = map_at_tail(dst, c.handle, c.bytes);
        if (st != KUN_OK) return st;
    }
    src->chunks.resize(first);
    src->mapped -= bytes;
    return KUN_OK;
}

int kun_vmm_region_shrink(kun_vmm_region* r, size_t bytes) {
    if (!r || bytes == 0) return KUN_ERR_INVALID_ARG;
    const size_t n = tail_chunks(r, bytes);
    if (n == 0) return KUN_ERR_MISALIGNED;
    for (size_t i = 0; i < n; ++i) {
        const kun_vmm_region::Chunk c = r->chunks.back();
        if (failed("hipMemUnmap", hipMemUnmap(r->base + r->mapped - c.bytes, c.bytes))) return KUN_ERR_HIP;
        r->chunks.pop_back();
        r->mapped -= c.bytes;
        if (failed("hipMemRelease", hipMemRelease(c.handle))) return KUN_ERR_HIP;
    }
    return KUN_OK;
}

int kun_vmm_region_destroy(kun_vmm_region* r) {
    if (!r) return KUN_OK;
    int st = KUN_OK;
    if (r->mapped > 0) st = kun_vmm_region_shrink(r, r->mapped);
    if (r->base && failed("hipMemAddressFree", hipMemAddressFree(r->base, r->reserved))) st = KUN_ERR_HIP;
    delete r;
    return st;
}

}  // extern "C"
