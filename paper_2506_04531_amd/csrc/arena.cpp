// Device memory sorted by HBM region, behind the C ABI (see include/halos.h, halos_arena_*).
//
// An MI355X hands a process its memory from a few large regions, one after the other, and a read-modify-write pass
// whose arrays sit in different regions gets about a fifth more bandwidth than one whose arrays share a region.
// Nothing in the HIP API says which region an allocation came from, so the arena finds out by measurement: it
// allocates 2 GiB slabs, times halos_probe_pair between a new slab and one representative slab per region found so
// far (slow = same region; the yardstick is a slab's two halves against each other), keeps the slabs each placement
// class needs and releases the rest.  Host logic only; the probe kernel is in kernels.hip.
#include "../../include/halos.h"
#include "../../include/halos_probe.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <new>
#include <numeric>
#include <vector>

namespace halos {
halos_status set_error(halos_status code, const char *fmt, ...);     // halos.cpp: fills the thread's error string
void register_handle(const void *h);                                 // halos.cpp: the registry of live handles
void unregister_handle(const void *h);
bool is_registered(const void *h);
}
using halos::set_error;

namespace {

constexpr uint32_t ARENA_MAGIC = 0x48415245u;   // "HARE"
constexpr uint64_t SLAB = 1ull << 31;
constexpr uint64_t HALF = 1ull << 30;
constexpr uint64_t ALIGN = 256;
constexpr double SAME_REGION_MARGIN = 1.08;     // a pair slower than margin x (a slab against itself) shares a region
constexpr int MAX_CLASSES = 8;

struct ClassState {
    std::vector<void *> slabs;      // region-sorted slabs first, overflow slabs (placed anywhere) after them
    size_t cursor_slab = 0;
    uint64_t cursor_off = 0;
    int region = -1;
};

}  // namespace

struct halos_arena {
    uint32_t magic = ARENA_MAGIC;
    int device = 0;
    int n_regions = 0;
    uint64_t walked = 0;
    double same_region_gbps = 0.0;
    std::vector<ClassState> cls;
    std::vector<void *> big;        // requests larger than a slab: allocations of their own
};

namespace {

struct Walk {                       // memory held during the search; whatever is left here at the end is released
    std::vector<std::vector<void *>> regions;
    std::vector<void *> ballast;    // slabs that straddle a region boundary
    ~Walk() {
        for (auto &r : regions) for (void *p : r) (void)hipFree(p);
        for (void *p : ballast) (void)hipFree(p);
    }
};

bool probe(void *a, void *b, double *gbps) {
    return halos_probe_pair(a, b, HALF, 2, nullptr, gbps) == HALOS_OK;
}

// Region index of the 1 GiB at p (regions.size() = none of the known ones); `first` is tried first.
int classify(const Walk &w, void *p, int first, double thr, bool *ok) {
    const int n = (int)w.regions.size();
    for (int k = -1; k < n; ++k) {
        const int r = k < 0 ? first : k;
        if (r < 0 || r >= n || (k >= 0 && r == first)) continue;
        double v = 0.0;
        if (!probe(w.regions[r][0], p, &v)) { *ok = false; return n; }
        if (v <= thr) return r;
    }
    return n;
}

}  // namespace

extern "C" {

halos_status halos_arena_create(int32_t n_classes, const uint64_t *bytes_per_class, uint64_t max_walk_bytes,
                                halos_arena **out) {
    if (!out) return set_error(HALOS_EINVAL, "out is NULL");
    *out = nullptr;
    if (n_classes < 1 || n_classes > MAX_CLASSES) return set_error(HALOS_EINVAL, "n_classes = %d outside 1..%d", n_classes, MAX_CLASSES);
    if (!bytes_per_class) return set_error(HALOS_EINVAL, "bytes_per_class is NULL");
    halos_arena *a = new (std::nothrow) halos_arena;
    if (!a) return set_error(HALOS_ENOMEM, "host allocation failed");
    hipError_t e = hipGetDevice(&a->device);
    size_t free_b = 0, total_b = 0;
    if (e == hipSuccess) e = hipMemGetInfo(&free_b, &total_b);
    if (e != hipSuccess) { delete a; return set_error(HALOS_EHIP, "querying the device: %s", hipGetErrorString(e)); }
    const uint64_t reserve = 8ull << 30;        // left alone for everybody else
    uint64_t budget = free_b > reserve ? free_b - reserve : 0;
    if (max_walk_bytes && max_walk_bytes < budget) budget = max_walk_bytes;

    // slabs wanted per class (+1: an allocation never straddles two slabs)
    std::vector<uint64_t> want(n_classes);
    for (int c = 0; c < n_classes; ++c) want[c] = bytes_per_class[c] ? (bytes_per_class[c] + SLAB - 1) / SLAB + 1 : 0;
    std::vector<uint64_t> want_sorted(want);
    std::sort(want_sorted.rbegin(), want_sorted.rend());

    Walk w;
    double thr = 0.0;
    int last = -1;
    bool ok = true;
    auto enough = [&] {
        std::vector<uint64_t> have;
        for (auto &r : w.regions) have.push_back(r.size());
        std::sort(have.rbegin(), have.rend());
        if ((int)have.size() < n_classes) return false;
        for (int c = 0; c < n_classes; ++c) if (have[c] < want_sorted[c]) return false;
        return true;
    };
    while (ok && a->walked + SLAB <= budget && !enough()) {
        void *slab = nullptr;
        e = hipMalloc(&slab, SLAB);
        if (e != hipSuccess) { (void)hipGetLastError(); break; }       // out of memory: work with what was found
        a->walked += SLAB;
        void *tail = static_cast<char *>(slab) + HALF;
        if (w.regions.empty()) {
            if (!probe(slab, tail, &a->same_region_gbps)) { (void)hipFree(slab); ok = false; break; }
            thr = SAME_REGION_MARGIN * a->same_region_gbps;
            w.regions.push_back({slab});
            last = 0;
            continue;
        }
        const int r_head = classify(w, slab, last, thr, &ok);
        const int r_tail = ok ? classify(w, tail, r_head < (int)w.regions.size() ? r_head : last, thr, &ok) : r_head;
        if (!ok) { (void)hipFree(slab); break; }
        if (r_head != r_tail) w.ballast.push_back(slab);
        else if (r_head == (int)w.regions.size()) { w.regions.push_back({slab}); last = r_head; }
        else { w.regions[r_head].push_back(slab); last = r_head; }
    }
    if (!ok) { delete a; return HALOS_EHIP; }      // the probe set the error string
    a->n_regions = (int)w.regions.size();

    // the largest classes get the regions with the most slabs; with fewer regions than classes, classes share
    std::vector<int> by_size(w.regions.size()), cls_order(n_classes);
    std::iota(by_size.begin(), by_size.end(), 0);
    std::iota(cls_order.begin(), cls_order.end(), 0);
    std::stable_sort(by_size.begin(), by_size.end(), [&](int x, int y) { return w.regions[x].size() > w.regions[y].size(); });
    std::stable_sort(cls_order.begin(), cls_order.end(), [&](int x, int y) { return want[x] > want[y]; });
    a->cls.resize(n_classes);
    for (int k = 0; k < n_classes && !by_size.empty(); ++k) {
        const int c = cls_order[k], r = by_size[k % by_size.size()];
        std::vector<void *> &src = w.regions[r];
        const size_t take = std::min<size_t>(src.size(), want[c]);
        a->cls[c].region = r;
        a->cls[c].slabs.assign(src.begin(), src.begin() + take);
        src.erase(src.begin(), src.begin() + take);
    }
    halos::register_handle(a);
    *out = a;
    return HALOS_OK;                               // ~Walk releases the slabs nobody took and the ballast
}

halos_status halos_arena_alloc(halos_arena *a, int32_t cls, uint64_t bytes, void **ptr) {
    if (!ptr) return set_error(HALOS_EINVAL, "ptr is NULL");
    *ptr = nullptr;
    if (!halos::is_registered(a) || a->magic != ARENA_MAGIC) return set_error(HALOS_EINVAL, "arena is not a valid handle");
    if (cls < 0 || cls >= (int)a->cls.size()) return set_error(HALOS_EINVAL, "class %d outside 0..%d", cls, (int)a->cls.size() - 1);
    if (bytes == 0) return set_error(HALOS_EINVAL, "bytes is 0");
    const uint64_t need = (bytes + ALIGN - 1) / ALIGN * ALIGN;
    if (need > SLAB) {                              // larger than a slab: its own allocation, wherever it lands
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, need);
        if (e != hipSuccess) { (void)hipGetLastError(); return set_error(HALOS_ENOMEM, "%llu bytes: %s", (unsigned long long)need, hipGetErrorString(e)); }
        a->big.push_back(p);
        *ptr = p;
        return HALOS_OK;
    }
    ClassState &c = a->cls[cls];
    if (c.cursor_slab < c.slabs.size() && c.cursor_off + need > SLAB) { c.cursor_slab += 1; c.cursor_off = 0; }
    if (c.cursor_slab >= c.slabs.size()) {          // the class has outgrown its region's slabs: take memory from anywhere
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, SLAB);
        if (e != hipSuccess) { (void)hipGetLastError(); return set_error(HALOS_ENOMEM, "overflow slab: %s", hipGetErrorString(e)); }
        c.slabs.push_back(p);
        c.cursor_slab = c.slabs.size() - 1;
        c.cursor_off = 0;
    }
    *ptr = static_cast<char *>(c.slabs[c.cursor_slab]) + c.cursor_off;
    c.cursor_off += need;
    return HALOS_OK;
}

halos_status halos_arena_info(const halos_arena *a, int32_t *n_regions, uint64_t *walked_bytes, double *same_region_gbps,
                              int32_t *region_of_class, int32_t *slabs_of_class) {
    if (!halos::is_registered(a) || a->magic != ARENA_MAGIC) return set_error(HALOS_EINVAL, "arena is not a valid handle");
    if (n_regions) *n_regions = a->n_regions;
    if (walked_bytes) *walked_bytes = a->walked;
    if (same_region_gbps) *same_region_gbps = a->same_region_gbps;
    for (size_t c = 0; c < a->cls.size(); ++c) {
        if (region_of_class) region_of_class[c] = a->cls[c].region;
        if (slabs_of_class) slabs_of_class[c] = (int32_t)a->cls[c].slabs.size();
    }
    return HALOS_OK;
}

void halos_arena_destroy(halos_arena *a) {
    if (!halos::is_registered(a) || a->magic != ARENA_MAGIC) return;
    halos::unregister_handle(a);
    (void)hipDeviceSynchronize();                  // nothing may still be running on memory that is about to go
    for (ClassState &c : a->cls) for (void *p : c.slabs) (void)hipFree(p);
    for (void *p : a->big) (void)hipFree(p);
    a->magic = 0;
    delete a;
}

}  // extern "C"
