// Host side of the library: the extensible KV block pool (range table), block resolution, and
// block-table validation.  No device work happens here.
//
// Section 4.1 ("Local instance memory management") extends the KVCache region at its tail with
// the physical memory of dropped parameters.  Here each extension is a separate byte range; block
// ids simply continue counting, so existing ids and addresses never change.
#include <limits.h>
#include <new>

#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "kun_internal.h"

namespace {
thread_local char g_hip_error[160] = "";

// One option from its textual value (NULL or "" = back to the default); false if the value is not valid.
bool apply_option(KunOptions& o, const char* name, const char* value) {
    const KunOptions dflt;
    const bool unset = !value || !value[0];
    if (!strcmp(name, "KUN_DECODE_PART")) {
        const int v = unset ? 0 : atoi(value);
        if (!unset && (v < 32 || v % 32 != 0)) return false;
        o.decode_part = v;
    } else if (!strcmp(name, "KUN_DECODE_WAVES")) {
        const int v = unset ? dflt.decode_waves : atoi(value);
        if (v != 1 && v != 2 && v != 4) return false;
        o.decode_waves = v;
    } else if (!strcmp(name, "KUN_DECODE_KERNEL")) {
        if (!unset && strcmp(value, "generic") && strcmp(value, "mfma")) return false;
        o.decode_generic = !unset && !strcmp(value, "generic");
    } else if (!strcmp(name, "KUN_DECODE_MAP")) {
        if (!unset && strcmp(value, "flat") && strcmp(value, "xcd")) return false;
        o.decode_flat_map = !unset && !strcmp(value, "flat");
    } else if (!strcmp(name, "KUN_DECODE_MERGE")) {
        if (unset || !strcmp(value, "auto")) o.decode_merge = 0;
        else if (!strcmp(value, "fold")) o.decode_merge = 1;
        else if (!strcmp(value, "kernel")) o.decode_merge = 2;
        else return false;
    } else if (!strcmp(name, "KUN_PREFILL_SHAPE")) {
        if (unset || !strcmp(value, "default")) o.prefill_shape = 0;
        else if (!strcmp(value, "persistent")) o.prefill_shape = 1;
        else if (!strcmp(value, "ring")) o.prefill_shape = 2;
        else if (!strcmp(value, "ring-persistent")) o.prefill_shape = 3;
        else return false;
    } else {
        return false;
    }
    return true;
}

const char* const kOptionNames[] = {"KUN_DECODE_PART", "KUN_DECODE_WAVES", "KUN_DECODE_KERNEL", "KUN_DECODE_MAP",
                                    "KUN_DECODE_MERGE", "KUN_PREFILL_SHAPE"};

KunOptions options_from_environment() {
    KunOptions o;
    for (const char* n : kOptionNames) (void)apply_option(o, n, getenv(n));   // invalid values are ignored
    return o;
}

KunOptions g_options = options_from_environment();
}

const KunOptions& kun_options() { return g_options; }

void kun_note_hip_error(const char* call, hipError_t e) {
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s (%d)", call, hipGetErrorString(e), (int)e);
}

extern "C" {

const char* kun_last_hip_error(void) { return g_hip_error; }

int kun_set_option(const char* name, const char* value) {
    if (!name) return KUN_ERR_INVALID_ARG;
    KunOptions o = g_options;
    if (!apply_option(o, name, value)) return KUN_ERR_INVALID_ARG;
    g_options = o;
    return KUN_OK;
}

const char* kun_status_string(int st) {
    switch (st) {
        case KUN_OK: return "KUN_OK";
        case KUN_ERR_INVALID_ARG: return "KUN_ERR_INVALID_ARG";
        case KUN_ERR_MISALIGNED: return "KUN_ERR_MISALIGNED";
        case KUN_ERR_TOO_SMALL: return "KUN_ERR_TOO_SMALL";
        case KUN_ERR_TOO_MANY_RANGES: return "KUN_ERR_TOO_MANY_RANGES";
        case KUN_ERR_BLOCK_OOB: return "KUN_ERR_BLOCK_OOB";
        case KUN_ERR_WORKSPACE: return "KUN_ERR_WORKSPACE";
        case KUN_ERR_HIP: return "KUN_ERR_HIP";
        case KUN_ERR_UNSUPPORTED: return "KUN_ERR_UNSUPPORTED";
        case KUN_ERR_OVERLAP: return "KUN_ERR_OVERLAP";
        case KUN_ERR_SCRATCH_LIMIT: return "KUN_ERR_SCRATCH_LIMIT";
        default: return "KUN_ERR_UNKNOWN";
    }
}

static int check_range(const kun_kv_pool* p, void* base, size_t bytes, int64_t* nblocks) {
    if (!base || bytes == 0) return KUN_ERR_INVALID_ARG;
    if (((uintptr_t)base & 255u) != 0) return KUN_ERR_MISALIGNED;
    int64_t nb = (int64_t)(bytes / p->block_bytes);
    if (nb < 1) return KUN_ERR_TOO_SMALL;
    if ((int64_t)p->ranges.first[p->ranges.n] + nb > (int64_t)INT32_MAX - 1) return KUN_ERR_INVALID_ARG;
    uintptr_t lo = (uintptr_t)base, hi = lo + bytes;
    for (int r = 0; r < p->ranges.n; ++r) {
        uintptr_t a = (uintptr_t)p->ranges.base[r], b = a + p->range_bytes[r];
        if (lo < b && a < hi) return KUN_ERR_OVERLAP;
    }
    *nblocks = nb;
    return KUN_OK;
}

int kun_kv_pool_create(kun_kv_pool** out, void* base, size_t bytes, int dtype, int num_kv_heads,
                       int head_dim, int block_size) {
    if (!out) return KUN_ERR_INVALID_ARG;
    *out = nullptr;
    if (dtype != KUN_F32 && dtype != KUN_BF16 && dtype != KUN_FP8_E4M3) return KUN_ERR_INVALID_ARG;
    if (num_kv_heads <= 0 || head_dim <= 0 || block_size <= 0) return KUN_ERR_INVALID_ARG;
    if ((block_size != 16 && block_size != 32 && block_size != 64 && block_size != 128) || (head_dim != 64 && head_dim != 128))
        return KUN_ERR_UNSUPPORTED;
    kun_kv_pool* p = new (std::nothrow) kun_kv_pool();
    if (!p) return KUN_ERR_INVALID_ARG;
    p->dtype = dtype;
    p->Hkv = num_kv_heads;
    p->d = head_dim;
    p->B = block_size;
    p->elt = dtype == KUN_F32 ? 4 : dtype == KUN_BF16 ? 2 : 1;
    p->page_bytes = (size_t)2 * block_size * head_dim * p->elt;
    p->block_bytes = p->page_bytes * num_kv_heads;
    p->ranges.n = 0;
    for (int i = 0; i <= KUN_MAX_RANGES; ++i) p->ranges.first[i] = INT32_MAX;
    for (int i = 0; i < KUN_MAX_RANGES; ++i) { p->ranges.base[i] = nullptr; p->range_bytes[i] = 0; }
    p->ranges.first[0] = 0;
    int64_t nb = 0;
    int st = check_range(p, base, bytes, &nb);
    if (st != KUN_OK) { delete p; return st; }
    p->ranges.base[0] = (char*)base;
    p->range_bytes[0] = bytes;
    p->ranges.first[1] = (int32_t)nb;
    p->ranges.n = 1;
    *out = p;
    return KUN_OK;
}

int kun_kv_pool_extend(kun_kv_pool* p, void* base, size_t bytes, int64_t* first_new_block,
                       int64_t* num_new_blocks) {
    if (!p) return KUN_ERR_INVALID_ARG;
    if (p->ranges.n >= KUN_MAX_RANGES) return KUN_ERR_TOO_MANY_RANGES;
    int64_t nb = 0;
    int st = check_range(p, base, bytes, &nb);
    if (st != KUN_OK) return st;
    int r = p->ranges.n;
    int32_t first = p->ranges.first[r];
    p->ranges.base[r] = (char*)base;
    p->range_bytes[r] = bytes;
    p->ranges.first[r + 1] = first + (int32_t)nb;
    p->ranges.n = r + 1;
    if (first_new_block) *first_new_block = first;
    if (num_new_blocks) *num_new_blocks = nb;
    return KUN_OK;
}

int kun_kv_pool_resize_tail(kun_kv_pool* p, size_t new_bytes, int64_t* first_changed_block,
                            int64_t* num_blocks_delta) {
    if (!p) return KUN_ERR_INVALID_ARG;
    const int r = p->ranges.n - 1;
    const int64_t nb = (int64_t)(new_bytes / p->block_bytes);
    if (nb < 1) return KUN_ERR_TOO_SMALL;
    const int64_t first = p->ranges.first[r], old_nb = (int64_t)p->ranges.first[r + 1] - first;
    if (first + nb > (int64_t)INT32_MAX - 1) return KUN_ERR_INVALID_ARG;
    uintptr_t lo = (uintptr_t)p->ranges.base[r], hi = lo + new_bytes;
    for (int i = 0; i < r; ++i) {
        uintptr_t a = (uintptr_t)p->ranges.base[i], b = a + p->range_bytes[i];
        if (lo < b && a < hi) return KUN_ERR_OVERLAP;
    }
    p->range_bytes[r] = new_bytes;
    p->ranges.first[r + 1] = (int32_t)(first + nb);
    if (first_changed_block) *first_changed_block = first + (nb < old_nb ? nb : old_nb);
    if (num_blocks_delta) *num_blocks_delta = nb - old_nb;
    return KUN_OK;
}

int kun_kv_pool_num_blocks(const kun_kv_pool* p, int64_t* n) {
    if (!p || !n) return KUN_ERR_INVALID_ARG;
    *n = p->ranges.first[p->ranges.n];
    return KUN_OK;
}

int kun_kv_pool_num_ranges(const kun_kv_pool* p, int* n) {
    if (!p || !n) return KUN_ERR_INVALID_ARG;
    *n = p->ranges.n;
    return KUN_OK;
}

int kun_kv_pool_block_bytes(const kun_kv_pool* p, size_t* bytes) {
    if (!p || !bytes) return KUN_ERR_INVALID_ARG;
    *bytes = p->block_bytes;
    return KUN_OK;
}

int kun_kv_pool_resolve(const kun_kv_pool* p, int64_t block, int* range, size_t* byte_off,
                        void** addr) {
    if (!p) return KUN_ERR_INVALID_ARG;
    if (block < 0 || block >= (int64_t)p->ranges.first[p->ranges.n]) return KUN_ERR_BLOCK_OOB;
    int r = 0;
    for (int i = 1; i < p->ranges.n; ++i)
        if (block >= p->ranges.first[i]) r = i;
    size_t off = (size_t)(block - p->ranges.first[r]) * p->block_bytes;
    if (range) *range = r;
    if (byte_off) *byte_off = off;
    if (addr) *addr = p->ranges.base[r] + off;
    return KUN_OK;
}

int kun_kv_pool_destroy(kun_kv_pool* p) {
    if (!p) return KUN_ERR_INVALID_ARG;
    delete p;
    return KUN_OK;
}

int kun_validate_block_table(const kun_kv_pool* p, const int32_t* table, int rows, int max_blocks,
                             const int32_t* ctx_len) {
    if (!p || rows < 0 || max_blocks < 0) return KUN_ERR_INVALID_ARG;
    if (rows > 0 && (!table || !ctx_len)) return KUN_ERR_INVALID_ARG;
    const int64_t nb = p->ranges.first[p->ranges.n];
    for (int s = 0; s < rows; ++s) {
        if (ctx_len[s] < 0) return KUN_ERR_INVALID_ARG;
        int64_t need = ((int64_t)ctx_len[s] + p->B - 1) / p->B;
        if (need > max_blocks) return KUN_ERR_INVALID_ARG;
        for (int64_t b = 0; b < need; ++b) {
            int32_t id = table[(size_t)s * max_blocks + b];
            if (id < 0 || id >= nb) return KUN_ERR_BLOCK_OOB;
        }
    }
    return KUN_OK;
}

}  // extern "C"
