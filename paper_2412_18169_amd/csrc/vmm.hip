// Virtual-memory form of the KVCache region (Section 4.1, "Local instance memory management"): one
// virtual address range is reserved for the largest KVCache the instance may ever hold, physical
// memory is mapped at its tail when the pool grows, and the physical chunks behind dropped
// parameters are remapped there without a copy (and back on restoration, Section 4.4).  Kernels then see ONE contiguous
// range whose size changes; kun_kv_pool_resize_tail tells the pool.
//
// Host code only (HIP virtual memory management API); no kernels.  The bookkeeping lives in
// vmm_region.h; this file supplies the HIP calls and the C entry points.
#include <new>

#include "kun_internal.h"
#include "vmm_region.h"

namespace {

constexpr size_t kMinGranularity = (size_t)2 << 20;

// 1 if the call failed (and notes it for kun_last_hip_error)
int failed(const char* call, hipError_t e) {
    if (e == hipSuccess) return 0;
    kun_note_hip_error(call, e);
    return 1;
}

struct HipVmm {
    typedef hipMemGenericAllocationHandle_t Handle;
    int device = 0;
    hipMemAllocationProp prop() const {
        hipMemAllocationProp p = {};
        p.type = hipMemAllocationTypePinned;
        p.location.type = hipMemLocationTypeDevice;
        p.location.id = device;
        return p;
    }
    int reserve(char** base, size_t bytes, size_t align) {
        void* va = nullptr;
        if (failed("hipMemAddressReserve", hipMemAddressReserve(&va, bytes, align, nullptr, 0))) return 1;
        *base = (char*)va;
        return 0;
    }
    int address_free(char* base, size_t bytes) { return failed("hipMemAddressFree", hipMemAddressFree(base, bytes)); }
    int create(Handle* h, size_t bytes) {
        const hipMemAllocationProp p = prop();
        return failed("hipMemCreate", hipMemCreate(h, bytes, &p, 0));
    }
    int release(Handle h) { return failed("hipMemRelease", hipMemRelease(h)); }
    int map(char* at, size_t bytes, Handle h) { return failed("hipMemMap", hipMemMap(at, bytes, 0, h, 0)); }
    int unmap(char* at, size_t bytes) { return failed("hipMemUnmap", hipMemUnmap(at, bytes)); }
    int set_access(char* base, size_t bytes) {
        hipMemAccessDesc acc = {};
        acc.location.type = hipMemLocationTypeDevice;
        acc.location.id = device;
        acc.flags = hipMemAccessFlagsProtReadWrite;
        return failed("hipMemSetAccess", hipMemSetAccess(base, bytes, &acc, 1));
    }
};

int to_status(int st) {
    switch (st) {
        case VMM_OK: return KUN_OK;
        case VMM_ERR_MISALIGNED: return KUN_ERR_MISALIGNED;
        case VMM_ERR_TOO_SMALL: return KUN_ERR_TOO_SMALL;
        case VMM_ERR_INVALID: return KUN_ERR_INVALID_ARG;
        default: return KUN_ERR_HIP;
    }
}

}  // namespace

struct kun_vmm_region {
    VmmRegion<HipVmm> r;
};

extern "C" {

int kun_vmm_region_create(kun_vmm_region** out, size_t reserve_bytes) {
    if (!out) return KUN_ERR_INVALID_ARG;
    *out = nullptr;
    if (reserve_bytes == 0) return KUN_ERR_INVALID_ARG;
    kun_vmm_region* reg = new (std::nothrow) kun_vmm_region();
    if (!reg) return KUN_ERR_INVALID_ARG;
    VmmRegion<HipVmm>& r = reg->r;
    if (failed("hipGetDevice", hipGetDevice(&r.drv.device))) { delete reg; return KUN_ERR_HIP; }
    const hipMemAllocationProp prop = r.drv.prop();
    if (failed("hipMemGetAllocationGranularity",
               hipMemGetAllocationGranularity(&r.gran, &prop, hipMemAllocationGranularityRecommended)) ||
        r.gran == 0) {
        delete reg;
        return KUN_ERR_HIP;
    }
    // The driver reports 4 KiB here; the region works in units of at least 2 MiB, base included, so
    // that chunks can be mapped with large pages.
    if (r.gran < kMinGranularity) r.gran = kMinGranularity;
    r.reserved = (reserve_bytes + r.gran - 1) / r.gran * r.gran;
    if (r.drv.reserve(&r.base, r.reserved, r.gran) != 0) {
        delete reg;
        return KUN_ERR_HIP;
    }
    *out = reg;
    return KUN_OK;
}

int kun_vmm_region_info(const kun_vmm_region* reg, void** base, size_t* mapped_bytes, size_t* reserved_bytes,
                        size_t* granularity) {
    if (!reg) return KUN_ERR_INVALID_ARG;
    if (base) *base = reg->r.base;
    if (mapped_bytes) *mapped_bytes = reg->r.mapped;
    if (reserved_bytes) *reserved_bytes = reg->r.reserved;
    if (granularity) *granularity = reg->r.gran;
    return KUN_OK;
}

int kun_vmm_region_grow(kun_vmm_region* reg, size_t bytes) {
    if (!reg) return KUN_ERR_INVALID_ARG;
    return to_status(reg->r.grow(bytes));
}

int kun_vmm_region_move_tail(kun_vmm_region* src, kun_vmm_region* dst, size_t bytes) {
    if (!src || !dst || src == dst) return KUN_ERR_INVALID_ARG;
    if (src->r.drv.device != dst->r.drv.device) return KUN_ERR_INVALID_ARG;
    return to_status(src->r.move_tail_to(dst->r, bytes));
}

int kun_vmm_region_shrink(kun_vmm_region* reg, size_t bytes) {
    if (!reg) return KUN_ERR_INVALID_ARG;
    return to_status(reg->r.shrink(bytes));
}

int kun_vmm_region_destroy(kun_vmm_region* reg) {
    if (!reg) return KUN_OK;
    const int st = to_status(reg->r.destroy());
    delete reg;
    return st;
}

}  // extern "C"
