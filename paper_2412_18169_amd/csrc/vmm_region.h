// Bookkeeping of a KVCache region that is ONE growing virtual address range (Section 4.1, "Local
// instance memory management"; Section 4.4 for the way back): which physical chunks are mapped where,
// and the order of driver calls that grows the range, hands its tail to another range without a copy,
// or gives it back.  The driver is a template parameter so that the bookkeeping -- in particular what
// both regions look like after a driver call fails half way -- can be exercised on the host with a
// driver that fails on demand; vmm.hip instantiates it with the HIP virtual-memory calls.
//
// Drv provides (all return 0 on success):
//   typedef Handle;
//   int reserve(char** base, size_t bytes, size_t align);     int address_free(char* base, size_t bytes);
//   int create(Handle* h, size_t bytes);                      int release(Handle h);
//   int map(char* at, size_t bytes, Handle h);                int unmap(char* at, size_t bytes);
//   int set_access(char* base, size_t bytes);                 (read/write for the region's device)
#pragma once

#include <stddef.h>

#include <vector>

enum {
    VMM_OK = 0, VMM_ERR_DRIVER = 1, VMM_ERR_MISALIGNED = 2, VMM_ERR_TOO_SMALL = 3, VMM_ERR_INVALID = 4,
    VMM_ERR_STUCK = 5      // map_at_tail only: the chunk is mapped and listed, but access could not be set
};

template <class Drv>
struct VmmRegion {
    struct Chunk {
        typename Drv::Handle handle;
        size_t bytes;
    };
    Drv drv;
    char* base = nullptr;
    size_t reserved = 0, mapped = 0, gran = 0;
    std::vector<Chunk> chunks;     // in address order; chunk i starts where chunk i-1 ends

    // Map `h` behind everything mapped so far.  Access is set for everything mapped so far, not for the
    // new chunk alone: asked for a chunk that is not the first of its reservation, the driver at hand
    // answers "invalid argument" unless all chunks have the same size (a call over [base, end of the
    // new chunk) never failed, for fresh and for remapped allocation handles).
    int map_at_tail(typename Drv::Handle h, size_t bytes) {
        if (mapped + bytes > reserved) return VMM_ERR_TOO_SMALL;
        char* at = base + mapped;
        if (drv.map(at, bytes, h) != 0) return VMM_ERR_DRIVER;
        int st = VMM_OK;
        if (drv.set_access(base, mapped + bytes) != 0) {
            if (drv.unmap(at, bytes) == 0) return VMM_ERR_DRIVER;
            st = VMM_ERR_STUCK;                    // it stays mapped, so it stays on the books
        }
        chunks.push_back({h, bytes});
        mapped += bytes;
        return st;
    }

    // Unmap the last chunk and forget it; the caller gets its handle (it is mapped nowhere then).
    int unmap_tail(Chunk* out) {
        const Chunk c = chunks.back();
        if (drv.unmap(base + mapped - c.bytes, c.bytes) != 0) return VMM_ERR_DRIVER;
        chunks.pop_back();
        mapped -= c.bytes;
        *out = c;
        return VMM_OK;
    }

    // number of tail chunks that make up exactly `bytes`; 0 if no whole number of chunks does
    size_t tail_chunks(size_t bytes) const {
        size_t n = 0, sum = 0;
        while (sum < bytes && n < chunks.size()) sum += chunks[chunks.size() - 1 - n++].bytes;
        return sum == bytes ? n : 0;
    }

    int grow(size_t bytes) {
        if (bytes == 0) return VMM_ERR_INVALID;
        if (bytes % gran != 0) return VMM_ERR_MISALIGNED;
        if (mapped + bytes > reserved) return VMM_ERR_TOO_SMALL;
        typename Drv::Handle h;
        if (drv.create(&h, bytes) != 0) return VMM_ERR_DRIVER;
        const int st = map_at_tail(h, bytes);
        if (st == VMM_ERR_STUCK) return VMM_ERR_DRIVER;
        if (st != VMM_OK) (void)drv.release(h);
        return st;
    }

    int shrink(size_t bytes) {
        if (bytes == 0) return VMM_ERR_INVALID;
        const size_t n = tail_chunks(bytes);
        if (n == 0) return VMM_ERR_MISALIGNED;
        for (size_t i = 0; i < n; ++i) {
            Chunk c;
            if (unmap_tail(&c) != VMM_OK) return VMM_ERR_DRIVER;
            if (drv.release(c.handle) != 0) return VMM_ERR_DRIVER;
        }
        return VMM_OK;
    }

    // Hand the last `bytes` of this region (whole chunks) to the tail of `dst`: same chunks, same order,
    // same contents, no copy.  The chunks are peeled off this region's tail, highest first, into a list
    // (this region stays a gapless range at every step) and then mapped at the destination lowest first
    // (the destination stays gapless too).  When a driver call fails, every
    // step already made is undone in reverse order, so that both regions are what they were; a chunk
    // that the driver then refuses to map back anywhere is released, and the regions still describe
    // exactly what is mapped: this region ends before the first chunk that could not be restored (the
    // chunks above it are released as well, a region cannot have a hole), the destination keeps the
    // chunks that arrived.
    int move_tail_to(VmmRegion& dst, size_t bytes) {
        if (&dst == this || bytes == 0) return VMM_ERR_INVALID;
        const size_t n = tail_chunks(bytes);
        if (n == 0) return VMM_ERR_MISALIGNED;
        if (dst.mapped + bytes > dst.reserved) return VMM_ERR_TOO_SMALL;
        std::vector<Chunk> moving;                 // highest chunk first
        moving.reserve(n);
        int st = VMM_OK;
        for (size_t i = 0; i < n && st == VMM_OK; ++i) {
            Chunk c;
            st = unmap_tail(&c);
            if (st == VMM_OK) moving.push_back(c);
        }
        size_t arrived = 0;
        while (st == VMM_OK && !moving.empty()) {
            st = dst.map_at_tail(moving.back().handle, moving.back().bytes);
            if (st == VMM_OK || st == VMM_ERR_STUCK) {
                moving.pop_back();
                ++arrived;
            }
        }
        if (st == VMM_OK) return VMM_OK;
        st = VMM_ERR_DRIVER;
        // undo: first what arrived at the destination (highest first, back onto `moving`), ...
        bool undone = true;
        while (arrived > 0 && undone) {
            Chunk c;
            if (dst.unmap_tail(&c) != VMM_OK) { undone = false; break; }
            moving.push_back(c);
            --arrived;
        }
        // ... then everything in `moving` back to this region's tail, lowest first
        while (undone && !moving.empty()) {
            const int back = map_at_tail(moving.back().handle, moving.back().bytes);
            if (back == VMM_OK || back == VMM_ERR_STUCK) moving.pop_back();
            if (back != VMM_OK) { undone = false; break; }
        }
        // the driver refused to undo: what is mapped nowhere goes back to the driver
        for (const Chunk& c : moving) (void)drv.release(c.handle);
        return st;
    }

    int destroy() {
        int st = VMM_OK;
        if (mapped > 0 && shrink(mapped) != VMM_OK) st = VMM_ERR_DRIVER;
        if (base && drv.address_free(base, reserved) != 0) st = VMM_ERR_DRIVER;
        base = nullptr;
        return st;
    }
};
