// csrc/cx_hbm.cpp against a model of device memory (the fake runtime declared in fake_hip/hip/hip_runtime.h):
// physical memory is handed out lowest address first, a handle's memory lives while the handle or a mapping of it
// does, and any call can be told to fail.  Checks the placement (every block spread evenly over what was free),
// the bookkeeping (fillers and handles released, nothing left after an error) and the error codes.
#include "cx_mix.h"
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <vector>

struct FakeHandle { size_t offset, size; bool alive; int maps; };

namespace fake {
constexpr size_t GiB = size_t{1} << 30, MiB = size_t{1} << 20;
size_t total = 288 * GiB, reported_extra = 0;            // hipMemGetInfo may over-report by reported_extra
std::map<size_t, size_t> free_list;                       // offset -> size, merged
std::set<FakeHandle *> handles;
std::map<char *, size_t> reservations;
struct Mapping { size_t size; FakeHandle *h; bool access; };
std::map<char *, Mapping> mappings;
int device = 0, syncs = 0, device_sets = 0;
long creates = 0, maps_done = 0, reserves = 0, accesses = 0;
long fail_create_at = -1, fail_create_from = -1, fail_map_at = -1, fail_reserve_at = -1, fail_access_at = -1;
char *next_va = reinterpret_cast<char *>(uintptr_t{1} << 44);

void reset(size_t used_at_start = 0)
{
    for (FakeHandle *h : handles) delete h;
    handles.clear(); reservations.clear(); mappings.clear(); free_list.clear();
    free_list[used_at_start] = total - used_at_start;
    reported_extra = 0; device = 0; syncs = device_sets = 0;
    creates = maps_done = reserves = accesses = 0;
    fail_create_at = fail_create_from = fail_map_at = fail_reserve_at = fail_access_at = -1;
}
size_t free_bytes() { size_t f = 0; for (auto &kv : free_list) f += kv.second; return f; }
void give_back(size_t off, size_t size)
{
    auto it = free_list.emplace(off, size).first;
    auto next = std::next(it);
    if (next != free_list.end() && it->first + it->second == next->first) { it->second += next->second; free_list.erase(next); }
    if (it != free_list.begin()) { auto prev = std::prev(it); if (prev->first + prev->second == it->first) { prev->second += it->second; free_list.erase(it); } }
}
void maybe_free(FakeHandle *h) { if (!h->alive && h->maps == 0) { give_back(h->offset, h->size); handles.erase(h); delete h; } }
}  // namespace fake

extern "C++" {
hipError_t hipGetDevice(int *d) { *d = fake::device; return hipSuccess; }
hipError_t hipSetDevice(int d) { fake::device = d; ++fake::device_sets; return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipDeviceSynchronize(void) { ++fake::syncs; return hipSuccess; }
hipError_t hipMemGetInfo(size_t *f, size_t *t) { *f = fake::free_bytes() + fake::reported_extra; *t = fake::total; return hipSuccess; }
hipError_t hipMemCreate(hipMemGenericAllocationHandle_t *out, size_t size, const hipMemAllocationProp *prop, unsigned long long)
{
    const long nth = fake::creates++;
    if (nth == fake::fail_create_at || (fake::fail_create_from >= 0 && nth >= fake::fail_create_from)) return hipErrorOutOfMemory;
    if (!prop || prop->type != hipMemAllocationTypePinned || prop->location.type != hipMemLocationTypeDevice || size == 0 || size % (2 * fake::MiB)) return hipErrorInvalidValue;
    size_t need = size, off = 0;                          // the model hands out memory in address order, split over gaps if it must
    for (auto &kv : fake::free_list) if (kv.second >= need) { off = kv.first; need = 0; break; }
    if (need) return hipErrorOutOfMemory;
    auto it = fake::free_list.find(off);
    const size_t rest = it->second - size;
    fake::free_list.erase(it);
    if (rest) fake::free_list[off + size] = rest;
    *out = new FakeHandle{off, size, true, 0};
    fake::handles.insert(*out);
    return hipSuccess;
}
hipError_t hipMemRelease(hipMemGenericAllocationHandle_t h)
{
    if (!fake::handles.count(h) || !h->alive) { std::printf("release of a dead handle\n"); std::exit(20); }
    h->alive = false; fake::maybe_free(h); return hipSuccess;
}
hipError_t hipMemAddressReserve(void **ptr, size_t size, size_t alignment, void *, unsigned long long)
{
    if (fake::reserves++ == fake::fail_reserve_at) return hipErrorOutOfMemory;
    if (size % (2 * fake::MiB) || alignment % (2 * fake::MiB)) return hipErrorInvalidValue;
    *ptr = fake::next_va; fake::reservations[fake::next_va] = size; fake::next_va += size + (64 * fake::MiB);
    return hipSuccess;
}
hipError_t hipMemAddressFree(void *ptr, size_t size)
{
    auto it = fake::reservations.find(static_cast<char *>(ptr));
    if (it == fake::reservations.end() || it->second != size) { std::printf("bad address free\n"); std::exit(21); }
    for (auto &m : fake::mappings) if (m.first >= it->first && m.first < it->first + size) { std::printf("address range freed while mapped\n"); std::exit(22); }
    fake::reservations.erase(it); return hipSuccess;
}
hipError_t hipMemMap(void *ptr, size_t size, size_t offset, hipMemGenericAllocationHandle_t h, unsigned long long)
{
    if (fake::maps_done++ == fake::fail_map_at) return hipErrorInvalidValue;
    char *p = static_cast<char *>(ptr);
    bool inside = false;
    for (auto &r : fake::reservations) inside |= p >= r.first && p + size <= r.first + r.second;
    if (!inside || offset != 0 || !fake::handles.count(h) || !h->alive || size != h->size || fake::mappings.count(p)) { std::printf("bad map\n"); std::exit(23); }
    fake::mappings[p] = {size, h, false}; ++h->maps; return hipSuccess;
}
hipError_t hipMemUnmap(void *ptr, size_t size)
{
    char *p = static_cast<char *>(ptr), *end = p + size;
    size_t covered = 0;
    for (auto it = fake::mappings.lower_bound(p); it != fake::mappings.end() && it->first < end;) {
        covered += it->second.size; --it->second.h->maps; fake::maybe_free(it->second.h); it = fake::mappings.erase(it);
    }
    if (covered != size) { std::printf("unmap of a range that is not exactly mapped pieces (%zu of %zu)\n", covered, size); std::exit(24); }
    return hipSuccess;
}
hipError_t hipMemSetAccess(void *ptr, size_t size, const hipMemAccessDesc *desc, size_t count)
{
    if (fake::accesses++ == fake::fail_access_at) return hipErrorInvalidValue;
    if (count != 1 || desc->flags != hipMemAccessFlagsProtReadWrite || desc->location.id != fake::device) return hipErrorInvalidValue;
    char *p = static_cast<char *>(ptr);
    for (auto &m : fake::mappings) if (m.first >= p && m.first < p + size) m.second.access = true;
    return hipSuccess;
}
}

#define CHECK(c) do { if (!(c)) { std::printf("line %d: %s\n", __LINE__, #c); return 1; } } while (0)
using fake::GiB; using fake::MiB;

static bool nothing_left() { return fake::mappings.empty() && fake::reservations.empty() && fake::handles.empty() && fake::free_list.size() == 1; }

// share of a block's bytes in each third of the memory that was free when the call started
static void thirds(void *base, size_t size, size_t lo, size_t hi, double out[3])
{
    out[0] = out[1] = out[2] = 0;
    char *p = static_cast<char *>(base);
    for (auto &m : fake::mappings)
        if (m.first >= p && m.first < p + size) {
            const double mid = static_cast<double>(m.second.h->offset) + 0.5 * m.second.size;
            out[std::min(2, static_cast<int>(3.0 * (mid - lo) / (hi - lo)))] += static_cast<double>(m.second.size) / size;
        }
}

int main()
{
    void *p[5];
    // 1. the C2 pair on an empty device: both blocks over all thirds, everything else free again
    fake::reset(2 * GiB);
    const int64_t c2 = int64_t{32} * 25558016 * 4;
    int64_t two[2] = {c2, c2};
    CHECK(cx_hbm_alloc(p, two, 2, 0) == CX_OK);
    const size_t c2r = (c2 + 2 * MiB - 1) / (2 * MiB) * (2 * MiB);
    CHECK(fake::free_bytes() == fake::total - 2 * GiB - 2 * c2r);          // fillers given back
    CHECK(fake::reservations.size() == 2 && fake::reservations.count(static_cast<char *>(p[0])) && fake::reservations[static_cast<char *>(p[1])] == c2r);
    for (FakeHandle *h : fake::handles) CHECK(!h->alive && h->maps == 1);   // handles released, memory held by the mappings
    size_t mapped = 0;
    for (auto &m : fake::mappings) { CHECK(m.second.access); CHECK(m.second.size % (2 * MiB) == 0 && m.second.size <= 256 * MiB); mapped += m.second.size; }
    CHECK(mapped == 2 * c2r && fake::mappings.size() == 2 * ((c2r + 256 * MiB - 1) / (256 * MiB)));
    for (int k = 0; k < 2; ++k) {
        double t[3]; thirds(p[k], c2r, 2 * GiB, fake::total, t);
        CHECK(t[0] > 0.25 && t[1] > 0.25 && t[2] > 0.25);
        size_t expect = 0;                                                   // pieces in address order without holes
        for (auto &m : fake::mappings) if (m.first >= static_cast<char *>(p[k]) && m.first < static_cast<char *>(p[k]) + c2r) { CHECK(m.first == static_cast<char *>(p[k]) + expect); expect += m.second.size; }
        CHECK(expect == c2r);
    }
    // a second call samples what is free now; freeing returns everything
    int64_t one[1] = {5 * int64_t(GiB) + 12345};
    CHECK(cx_hbm_alloc(p + 2, one, 1, 0) == CX_OK);
    { double t[3]; thirds(p[2], 5 * GiB + 2 * MiB, 2 * GiB, fake::total, t); CHECK(t[0] > 0.25 && t[1] > 0.25 && t[2] > 0.25); }
    fake::device = 3;                                                        // freed from another current device
    CHECK(cx_hbm_free(p[0]) == CX_OK && fake::device == 3 && fake::device_sets == 2 && fake::syncs == 1);
    fake::device = 0;
    CHECK(cx_hbm_free(p[0]) == CX_ERR_UNSUPPORTED);
    CHECK(cx_hbm_free(static_cast<char *>(p[1]) + 2 * MiB) == CX_ERR_UNSUPPORTED);
    CHECK(cx_hbm_free(p[1]) == CX_OK && cx_hbm_free(p[2]) == CX_OK);
    CHECK(nothing_left() && fake::free_bytes() == fake::total - 2 * GiB);

    // 2. the driver reports more free memory than it can give: the fillers run out, the blocks are still served
    fake::reset(200 * GiB);
    fake::reported_extra = 60 * GiB;
    CHECK(cx_hbm_alloc(p, two, 2, 0) == CX_OK);
    CHECK(fake::free_bytes() == fake::total - 200 * GiB - 2 * c2r);
    CHECK(cx_hbm_free(p[0]) == CX_OK && cx_hbm_free(p[1]) == CX_OK && nothing_left());

    // 3. more asked for than is free; a nearly full device (no room for fillers) still serves what fits
    fake::reset(286 * GiB);
    int64_t big[1] = {3 * int64_t(GiB)};
    CHECK(cx_hbm_alloc(p, big, 1, 0) == CX_ERR_MEMORY && p[0] == nullptr && nothing_left());
    int64_t fits[1] = {int64_t(GiB) + 1};
    CHECK(cx_hbm_alloc(p, fits, 1, 0) == CX_OK && fake::free_bytes() == 2 * GiB - (GiB + 2 * MiB));
    CHECK(cx_hbm_free(p[0]) == CX_OK && nothing_left());

    // 4. every runtime call fails once, at every position: an error code, NULL pointers, nothing left behind
    int64_t three[3] = {700 * int64_t(MiB), 2 * int64_t(MiB), 300 * int64_t(MiB) + 1};          // 3 + 1 + 2 pieces
    fake::reset(); CHECK(cx_hbm_alloc(p, three, 3, 0) == CX_OK);
    const long n_create = fake::creates, n_map = fake::maps_done, n_reserve = fake::reserves, n_access = fake::accesses;
    CHECK(n_map == 6 && n_reserve == 3 && n_access == 3 && n_create > 6);
    for (int k = 0; k < 3; ++k) CHECK(cx_hbm_free(p[k]) == CX_OK);
    CHECK(nothing_left());
    for (long at = 0; at < n_create; ++at) {
        // one creation fails: a filler (no more skipping) or a piece (the fillers are given back and it is tried again)
        fake::reset(); fake::fail_create_at = at;
        CHECK(cx_hbm_alloc(p, three, 3, 0) == CX_OK);
        for (int k = 0; k < 3; ++k) CHECK(cx_hbm_free(p[k]) == CX_OK);
        CHECK(nothing_left());
        // every creation from here on fails: out of memory, nothing left behind
        fake::reset(); fake::fail_create_from = at;
        p[0] = p[1] = p[2] = reinterpret_cast<void *>(1);
        CHECK(cx_hbm_alloc(p, three, 3, 0) == CX_ERR_MEMORY && !p[0] && !p[1] && !p[2]);
        CHECK(nothing_left());
    }
    for (long at = 0; at < n_map; ++at) { fake::reset(); fake::fail_map_at = at; CHECK(cx_hbm_alloc(p, three, 3, 0) == CX_ERR_HIP && !p[0] && !p[2] && nothing_left()); }
    for (long at = 0; at < n_reserve; ++at) { fake::reset(); fake::fail_reserve_at = at; CHECK(cx_hbm_alloc(p, three, 3, 0) == CX_ERR_HIP && !p[1] && nothing_left()); }
    for (long at = 0; at < n_access; ++at) { fake::reset(); fake::fail_access_at = at; CHECK(cx_hbm_alloc(p, three, 3, 0) == CX_ERR_HIP && !p[0] && nothing_left()); }

    // 5. 64 blocks at once, and the argument errors
    fake::reset();
    std::vector<int64_t> many(64, 300 * int64_t(MiB));
    std::vector<void *> q(64);
    CHECK(cx_hbm_alloc(q.data(), many.data(), 64, 0) == CX_OK);
    CHECK(std::set<void *>(q.begin(), q.end()).size() == 64);
    for (void *b : q) CHECK(cx_hbm_free(b) == CX_OK);
    CHECK(nothing_left());
    CHECK(cx_hbm_alloc(nullptr, two, 2, 0) == CX_ERR_NULL && cx_hbm_alloc(p, nullptr, 2, 0) == CX_ERR_NULL);
    CHECK(cx_hbm_alloc(p, two, 0, 0) == CX_ERR_SHAPE && cx_hbm_alloc(p, two, 65, 0) == CX_ERR_SHAPE && cx_hbm_alloc(p, two, 2, 4) == CX_ERR_UNSUPPORTED);
    int64_t bad[2] = {c2, 0};
    CHECK(cx_hbm_alloc(p, bad, 2, 0) == CX_ERR_SHAPE && cx_hbm_free(nullptr) == CX_ERR_NULL);
    CHECK(fake::creates == 0 || nothing_left());
    fake::reset();
    std::printf("ok\n");
    return 0;
}
