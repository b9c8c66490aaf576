// Host-only check of the KVCache-region bookkeeping (paper_2412_18169_amd/csrc/vmm_region.h) with a
// driver that models the address space and fails the n-th call on demand: whatever call fails during
// move_tail_to, grow or shrink, both regions must list exactly what the model has mapped, no handle
// may be lost or released twice, and when the failed step could be undone both regions must be what
// they were.  Built and run by tests/test_host_boundary.py with g++; prints "vmm bookkeeping ok".
#include <stdio.h>
#include <stdlib.h>

#include <map>
#include <set>
#include <vector>

#include "vmm_region.h"

struct World {
    std::map<char*, std::pair<size_t, int>> mapped;    // address -> (bytes, handle)
    std::set<int> alive;                               // handles created and not released
    int next_handle = 1;
    long calls = 0, fail_from = -1, fail_count = 0;    // calls number fail_from .. fail_from + fail_count - 1 fail
    bool fails() {
        const long c = calls++;
        return fail_from >= 0 && c >= fail_from && c < fail_from + fail_count;
    }
};
static World* W;

#define CHECK(x) do { if (!(x)) { printf("FAILED %s (line %d)\n", #x, __LINE__); exit(1); } } while (0)

struct MockDrv {
    typedef int Handle;
    int reserve(char** base, size_t, size_t) { *base = (char*)0x100000000; return 0; }
    int address_free(char*, size_t) { return 0; }
    int create(Handle* h, size_t) {
        if (W->fails()) return 1;
        *h = W->next_handle++;
        W->alive.insert(*h);
        return 0;
    }
    int release(Handle h) {
        CHECK(W->alive.count(h) == 1);                 // never released twice
        for (auto& m : W->mapped) CHECK(m.second.second != h);   // never released while mapped
        W->alive.erase(h);
        return 0;                                      // (a release that fails would only leak)
    }
    int map(char* at, size_t bytes, Handle h) {
        if (W->fails()) return 1;
        CHECK(W->alive.count(h) == 1);
        for (auto& m : W->mapped) {
            CHECK(m.second.second != h);               // a handle is mapped at most once
            CHECK(at + bytes <= m.first || m.first + m.second.first <= at);   // no overlap
        }
        W->mapped[at] = {bytes, h};
        return 0;
    }
    int unmap(char* at, size_t bytes) {
        if (W->fails()) return 1;
        auto it = W->mapped.find(at);
        CHECK(it != W->mapped.end() && it->second.first == bytes);   // only what is mapped, as a whole
        W->mapped.erase(it);
        return 0;
    }
    int set_access(char*, size_t) { return W->fails() ? 1 : 0; }
};

typedef VmmRegion<MockDrv> Region;

static void init(Region& r, char* base, size_t reserved) {
    r.base = base;
    r.reserved = reserved;
    r.gran = 4096;
}

// The regions list exactly what the model has mapped, gapless from their bases; nothing else is alive.
static void check_consistent(const Region& a, const Region& b) {
    size_t n = 0;
    std::set<int> listed;
    for (const Region* r : {&a, &b}) {
        size_t off = 0;
        for (auto& c : r->chunks) {
            auto it = W->mapped.find(r->base + off);
            CHECK(it != W->mapped.end() && it->second.first == c.bytes && it->second.second == c.handle);
            listed.insert(c.handle);
            off += c.bytes;
            ++n;
        }
        CHECK(off == r->mapped && r->mapped <= r->reserved);
    }
    CHECK(n == W->mapped.size());
    CHECK(listed == W->alive);
}

static std::vector<std::pair<int, size_t>> snapshot(const Region& r) {
    std::vector<std::pair<int, size_t>> v;
    for (auto& c : r.chunks) v.push_back({c.handle, c.bytes});
    return v;
}

int main() {
    const size_t K = 4096;
    const size_t src_sizes[] = {2 * K, K, 3 * K, K, 2 * K};      // move the last three: 6 K
    long cases = 0, undone = 0, degraded = 0;
    for (long fail_count = 0; fail_count <= 12; ++fail_count) {
        for (long fail_at = 0; fail_at < 40; ++fail_at) {
            World world;
            W = &world;
            Region src, dst;
            init(src, (char*)0x100000000, 64 * K);
            init(dst, (char*)0x200000000, 64 * K);
            for (size_t s : src_sizes) CHECK(src.grow(s) == VMM_OK);
            CHECK(dst.grow(K) == VMM_OK);
            CHECK(dst.grow(2 * K) == VMM_OK);
            check_consistent(src, dst);
            const auto src0 = snapshot(src), dst0 = snapshot(dst);
            // argument errors change nothing
            CHECK(src.move_tail_to(dst, 5 * K) == VMM_ERR_MISALIGNED);   // not a whole number of chunks
            CHECK(src.move_tail_to(dst, 0) == VMM_ERR_INVALID && src.move_tail_to(src, 2 * K) == VMM_ERR_INVALID);
            CHECK(snapshot(src) == src0 && snapshot(dst) == dst0);
            world.calls = 0;
            world.fail_from = fail_count ? fail_at : -1;
            world.fail_count = fail_count;
            const int st = src.move_tail_to(dst, 6 * K);
            const long used = world.calls;
            world.fail_from = -1;
            check_consistent(src, dst);
            ++cases;
            if (st == VMM_OK) {
                CHECK(fail_count == 0 || fail_at >= used);
                CHECK(src.mapped == 3 * K && dst.mapped == 9 * K);
                auto d = snapshot(dst);                    // same chunks, same order, behind what dst had
                CHECK(d.size() == 5 && d[2] == src0[2] && d[3] == src0[3] && d[4] == src0[4]);
                // and back again (restoration)
                CHECK(dst.move_tail_to(src, 6 * K) == VMM_OK);
                CHECK(snapshot(src) == src0 && snapshot(dst) == dst0);
            } else {
                CHECK(st == VMM_ERR_DRIVER);
                if (snapshot(src) == src0 && snapshot(dst) == dst0) ++undone;
                else {
                    // the driver also refused the undoing: src is a prefix of what it was, dst what it was
                    // plus some of the moved chunks in order, the others were released
                    ++degraded;
                    auto s = snapshot(src), d = snapshot(dst);
                    CHECK(s.size() <= src0.size() && d.size() >= dst0.size());
                    for (size_t i = 0; i < s.size(); ++i) CHECK(s[i] == src0[i]);
                    for (size_t i = 0; i < d.size(); ++i) CHECK(d[i] == (i < 2 ? dst0[i] : src0[i]));
                }
                if (fail_count == 1) CHECK(snapshot(src) == src0 && snapshot(dst) == dst0);   // one failure is always undone
            }
            // the regions stay usable: grow and shrink still work on both, then everything goes back
            CHECK(src.grow(K) == VMM_OK && dst.grow(K) == VMM_OK);
            check_consistent(src, dst);
            CHECK(src.shrink(K) == VMM_OK);
            CHECK(src.destroy() == VMM_OK && dst.destroy() == VMM_OK);
            CHECK(world.mapped.empty() && world.alive.empty());
        }
    }
    // grow: a failing create, map or set_access leaves the region as it was and leaks nothing
    for (long fail_at = 0; fail_at < 3; ++fail_at) {
        World world;
        W = &world;
        Region r, other;
        init(r, (char*)0x100000000, 8 * K);
        init(other, (char*)0x200000000, 8 * K);
        CHECK(r.grow(2 * K) == VMM_OK);
        world.calls = 0;
        world.fail_from = fail_at;
        world.fail_count = 1;
        CHECK(r.grow(K) == VMM_ERR_DRIVER);
        world.fail_from = -1;
        check_consistent(r, other);
        CHECK(r.mapped == 2 * K && r.grow(100) == VMM_ERR_MISALIGNED && r.grow(8 * K) == VMM_ERR_TOO_SMALL);
        CHECK(r.destroy() == VMM_OK);
    }
    printf("vmm bookkeeping ok: %ld cases, %ld undone, %ld degraded\n", cases, undone, degraded);
    return undone > 0 && degraded > 0 ? 0 : 1;
}
