// C ABI of the HALoS server-side update path (see include/halos.h for the contract of every call).
// This file is host logic only: argument checking, the protocol state machine, the small device
// tables, and the decision which kernel to launch.  All parameter arithmetic is in kernels.hip.
#include "../../include/halos.h"
#include "../../include/halos_probe.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <unordered_set>
#include <vector>

#include "kernels.hpp"
#include "protocol.hpp"

using namespace halos;

namespace {
thread_local std::string g_last_error;
}

namespace halos {
// Shared with the other translation units of the library: record the calling thread's error text, return `code`.
halos_status set_error(halos_status code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

// Handles (servers and arenas) are validated against a registry of live ones, so that a stale or foreign pointer is
// rejected without being dereferenced.  Shared with the other translation units of the library.
namespace {
std::mutex g_registry_mutex;
std::unordered_set<const void *> g_live_handles;
}
void register_handle(const void *h) { std::lock_guard<std::mutex> lk(g_registry_mutex); g_live_handles.insert(h); }
void unregister_handle(const void *h) { std::lock_guard<std::mutex> lk(g_registry_mutex); g_live_handles.erase(h); }
bool is_registered(const void *h) {
    if (!h) return false;
    std::lock_guard<std::mutex> lk(g_registry_mutex);
    return g_live_handles.count(h) != 0;
}
}  // namespace halos

namespace {

#define fail(...) halos::set_error(__VA_ARGS__)

halos_status fail_hip(hipError_t e, const char *what) {
    return fail(HALOS_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// One workgroup per compute unit = one wavefront per SIMD: measured best on MI355X (more resident wavefronts only
// deepen the queues in front of the memory controllers; 1-4 % slower at 2..32 per compute unit on every workload).
std::atomic<int> g_blocks_per_cu{1};
std::atomic<int> g_nontemporal{1};

constexpr uint32_t GPS_MAGIC = 0x48475053u;   // "HGPS"
constexpr uint32_t LPS_MAGIC = 0x484c5053u;   // "HLPS"


bool rule_ok(const halos_rule &r) {
    return std::isfinite(r.eta) && std::isfinite(r.beta) && std::isfinite(r.cg);
}

halos_status check_hparams(const halos_hparams *hp) {
    if (!hp) return fail(HALOS_EINVAL, "hparams is NULL");
    if (!rule_ok(hp->local) || !rule_ok(hp->global)) return fail(HALOS_EINVAL, "non-finite eta/beta/cg");
    if (!(hp->alpha >= 0.0f && hp->alpha <= 1.0f)) return fail(HALOS_EINVAL, "alpha %g outside [0,1]", (double)hp->alpha);
    if (hp->K < 1) return fail(HALOS_EINVAL, "K = %d, must be >= 1", hp->K);
    if ((hp->flags & ~(uint32_t)(HALOS_FLAG_NORMS | HALOS_FLAG_SNAPSHOT | HALOS_FLAG_GPS_NO_MOMENTUM | HALOS_FLAG_DEFER_CLEAR |
                                 HALOS_FLAG_BF16_MOMENTUM)) != 0)
        return fail(HALOS_EINVAL, "unknown bits in flags");
    if ((hp->flags & HALOS_FLAG_SNAPSHOT) && (hp->flags & HALOS_FLAG_DEFER_CLEAR))
        return fail(HALOS_EINVAL, "HALOS_FLAG_DEFER_CLEAR has no meaning under HALOS_FLAG_SNAPSHOT (the merge writes the snapshot)");
    if ((hp->flags & HALOS_FLAG_GPS_NO_MOMENTUM) && hp->global.beta != 0.0f)
        return fail(HALOS_EINVAL, "HALOS_FLAG_GPS_NO_MOMENTUM needs global.beta = 0, got %g", (double)hp->global.beta);
    return HALOS_OK;
}

}  // namespace

struct halos_gps {
    uint32_t magic = GPS_MAGIC;
    int device = 0;
    int n_cu = 1;
    std::vector<int64_t> numel;
    int64_t total = 0;
    std::vector<TileRange> ranges;
    Tile *d_tiles = nullptr;
    uint32_t n_tiles = 0;
    void *d_tables = nullptr;          // one allocation: [Theta pointers | M pointers]
    float **d_Theta = nullptr, **d_M = nullptr;
    float **d_buffer = nullptr;        // gradient buffer of the delayed momentum (third table of d_tables; null until set)
    MomentumCycle cycle;
    halos_rule rule{};
    halos_hparams hp{};
    int64_t updates = 0;
    int n_lps_attached = 0;
    bool no_momentum = false;          // HALOS_FLAG_GPS_NO_MOMENTUM: there is no M; beta stays 0
    bool momentum_bf16 = false;        // HALOS_FLAG_BF16_MOMENTUM: M and every local server's m hold bfloat16
    std::vector<const void *> validated_delta;   // last pointer set accepted by halos_gps_push_update
    halos_dtype validated_delta_dtype = HALOS_F32;
    bool retired = false;              // halos_gps_destroy was called while local servers were still attached
};

struct PendingDelta {
    std::vector<const void *> ptrs;
    halos_dtype dtype = HALOS_F32;
    bool end_model = false;            // ptrs hold the worker's end model, not a pseudo-gradient
    uint32_t staleness = 0;
    float weight = 1.0f;               // the caller's scalar on this delta
};

struct halos_lps {
    uint32_t magic = LPS_MAGIC;
    halos_gps *gps = nullptr;
    int32_t id = 0;
    void *d_tables = nullptr;          // one allocation: [theta | m | acc] pointer tables
    float **d_theta = nullptr, **d_m = nullptr, **d_acc = nullptr;
    float **d_worker_model = nullptr;  // n_workers tables of n_tensors pointers, appended to d_tables
    float **d_buffer = nullptr;        // gradient buffer of the delayed momentum (a table of d_tables; null until set)
    float **d_delta = nullptr;         // n_workers tables of delta pointers, for the passes that take several deltas
    std::vector<std::vector<const void *>> delta_in_table;   // per worker: the pointer set its device table holds now
    MomentumCycle cycle;
    std::vector<char> worker_has_model;
    std::vector<std::vector<const void *>> worker_model_host;   // per worker: the registered model buffers (host copy)
    // update-norm monitors (HALOS_FLAG_NORMS): per-workgroup partial sums, then [ |g|^2 of the last update,
    // |theta - Theta_i|^2 before the last merge ]
    double *d_norm_partials = nullptr;
    double *d_norm_results = nullptr;
    uint32_t norm_partial_cap = 0;
    halos_rule rule{};
    float alpha = 0.f;
    bool snapshot = false;             // third buffer holds theta_{t_last}; Delta is formed by subtraction at the send
    bool defer_clear = false;          // HALOS_FLAG_DEFER_CLEAR: merges leave the third buffer as it is ...
    bool third_stale = false;          // ... and the next accumulating update restarts it (set by a merge, cleared by that update)
    LpsProtocol proto;
    std::vector<PendingDelta> pending;           // per worker: the delta it has queued
    std::vector<std::vector<const void *>> validated;   // per worker: last pointer set whose ranges were checked
    std::vector<halos_dtype> validated_dtype;
    std::vector<const void *> validated_pull;
    const void *validated_norm_out = nullptr;    // last device pointer accepted by halos_lps_step_norms
    uint32_t max_staleness = 0;
    halos_lps(int32_t n_workers, int32_t K) : proto(n_workers, K) {}
};

namespace {

bool live_gps(const halos_gps *g) { return is_registered(g) && g->magic == GPS_MAGIC && !g->retired; }
bool live_lps(const halos_lps *l) { return is_registered(l) && l->magic == LPS_MAGIC; }

static_assert(POS_FIRST == CYCLE_FIRST && POS_INNER == CYCLE_INNER && POS_REFRESH == CYCLE_REFRESH,
              "the protocol's cycle positions are the kernels' rule selectors");

LaunchShape current_shape(const halos_gps *g) {
    LaunchShape s;
    s.grid_cap = g_blocks_per_cu.load() * g->n_cu;
    s.nontemporal = g_nontemporal.load() != 0;
    return s;
}

// Each non-empty tensor must be a 16-byte aligned device address with room for numel elements.
halos_status check_tensors(const halos_gps *g, const void *const *ptrs, size_t elem_bytes, const char *what) {
    if (!ptrs) return fail(HALOS_EINVAL, "%s: pointer array is NULL", what);
    for (size_t i = 0; i < g->numel.size(); ++i) {
        if (g->numel[i] == 0) continue;
        const void *p = ptrs[i];
        if (!p) return fail(HALOS_EINVAL, "%s: tensor %zu is NULL", what, i);
        if ((reinterpret_cast<uintptr_t>(p) & 15u) != 0)
            return fail(HALOS_EINVAL, "%s: tensor %zu is not 16-byte aligned", what, i);
        hipPointerAttribute_t attr;
        hipError_t e = hipPointerGetAttributes(&attr, p);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(HALOS_EINVAL, "%s: tensor %zu is not a device pointer (%s)", what, i, hipGetErrorString(e));
        }
        if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged)
            return fail(HALOS_EINVAL, "%s: tensor %zu is not device memory", what, i);
        if (attr.type == hipMemoryTypeDevice && attr.device != g->device)
            return fail(HALOS_EINVAL, "%s: tensor %zu lives on device %d, server on %d", what, i, attr.device, g->device);
        hipDeviceptr_t base = nullptr;
        size_t size = 0;
        e = hipMemGetAddressRange(&base, &size, const_cast<void *>(p));
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(HALOS_EINVAL, "%s: tensor %zu: cannot query its allocation (%s)", what, i, hipGetErrorString(e));
        }
        const uintptr_t end = reinterpret_cast<uintptr_t>(p) + (size_t)g->numel[i] * elem_bytes;
        if (end > reinterpret_cast<uintptr_t>(base) + size)
            return fail(HALOS_EINVAL, "%s: tensor %zu (%lld elements) runs past the end of its allocation", what, i,
                        (long long)g->numel[i]);
    }
    return HALOS_OK;
}

halos_status check_device(const halos_gps *g) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev != g->device) return fail(HALOS_EINVAL, "current device %d differs from the server's device %d", dev, g->device);
    return HALOS_OK;
}

void fill_args(PtrArgs &a, const void *const *ptrs, const TileRange &r, size_t n_tensors) {
    for (int i = 0; i < MAX_ARG_TENSORS; ++i) {
        const size_t t = (size_t)r.tensor_base + i;
        a.p[i] = t < n_tensors ? ptrs[t] : nullptr;
    }
}

halos_status upload_tables(void **d_out, const std::vector<const void *const *> &host_tabs, size_t n_tensors,
                           size_t extra_null_tables = 0) {
    const size_t bytes = (host_tabs.size() + extra_null_tables) * n_tensors * sizeof(void *);
    void *d = nullptr;
    hipError_t e = hipMalloc(&d, bytes ? bytes : sizeof(void *));
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(HALOS_ENOMEM, "pointer tables: %s", hipGetErrorString(e)); }
    std::vector<const void *> flat;
    flat.reserve((host_tabs.size() + extra_null_tables) * n_tensors);
    for (const void *const *tab : host_tabs)
        for (size_t i = 0; i < n_tensors; ++i) flat.push_back(tab[i]);
    flat.resize((host_tabs.size() + extra_null_tables) * n_tensors, nullptr);
    if (bytes) {
        e = hipMemcpy(d, flat.data(), bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) { (void)hipFree(d); return fail_hip(e, "uploading pointer tables"); }
    }
    *d_out = d;
    return HALOS_OK;
}

// A probe buffer must be 16-byte aligned device memory with room for `used` bytes.
halos_status check_probe_buffer(const void *p, uint64_t used) {
    if (!p) return fail(HALOS_EINVAL, "NULL buffer");
    if ((reinterpret_cast<uintptr_t>(p) & 15u) != 0) return fail(HALOS_EINVAL, "buffers must be 16-byte aligned");
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess || (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged)) {
        (void)hipGetLastError();
        return fail(HALOS_EINVAL, "not a device pointer");
    }
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    e = hipMemGetAddressRange(&base, &size, const_cast<void *>(p));
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(HALOS_EINVAL, "cannot query the allocation"); }
    if (reinterpret_cast<uintptr_t>(p) + used > reinterpret_cast<uintptr_t>(base) + size)
        return fail(HALOS_EINVAL, "buffer is smaller than `bytes`");
    return HALOS_OK;
}

// Run `launch` once untimed and `reps` times between two events on stream s; *ms = elapsed time of the timed part.
template <class Launch>
halos_status time_launches(hipStream_t s, int reps, Launch launch, float *ms) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e != hipSuccess) { if (e0) (void)hipEventDestroy(e0); return fail_hip(e, "hipEventCreate"); }
    e = launch();
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    for (int r = 0; r < reps && e == hipSuccess; ++r) e = launch();
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    *ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail_hip(e, "timing the probe");
    return HALOS_OK;
}

}  // namespace

extern "C" {

const char *halos_last_error(void) { return g_last_error.c_str(); }

halos_rule halos_paper_rule(float eta, float beta) {
    halos_rule r;
    r.eta = eta;
    r.beta = beta;
    r.cg = 1.0f - beta;
    return r;
}

halos_status halos_set_launch_config(int32_t blocks_per_cu, int32_t nontemporal) {
    if (blocks_per_cu < 0 || blocks_per_cu > 64) return fail(HALOS_EINVAL, "blocks_per_cu %d outside 0..64", blocks_per_cu);
    if (nontemporal < -1 || nontemporal > 1) return fail(HALOS_EINVAL, "nontemporal %d outside -1..1", nontemporal);
    if (blocks_per_cu > 0) g_blocks_per_cu.store(blocks_per_cu);
    if (nontemporal >= 0) g_nontemporal.store(nontemporal);
    return HALOS_OK;
}

halos_status halos_probe_pair(void *a, void *b, uint64_t bytes, int32_t reps, void *stream, double *gbps) {
    if (!a || !b || !gbps) return fail(HALOS_EINVAL, "NULL argument");
    if (((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15u) != 0)
        return fail(HALOS_EINVAL, "buffers must be 16-byte aligned");
    const uint64_t tile_bytes = (uint64_t)TILE_ELEMS * sizeof(float);
    if (bytes < tile_bytes) return fail(HALOS_EINVAL, "bytes = %llu, must be >= %llu", (unsigned long long)bytes,
                                        (unsigned long long)tile_bytes);
    if (reps < 1 || reps > 1000) return fail(HALOS_EINVAL, "reps = %d outside 1..1000", reps);
    const uint64_t n_tiles64 = bytes / tile_bytes;
    if (n_tiles64 > 0xFFFFFFFFull) return fail(HALOS_EINVAL, "bytes too large");
    const uint64_t used = n_tiles64 * tile_bytes;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    if ((pa <= pb && pa + used > pb) || (pb <= pa && pb + used > pa)) return fail(HALOS_EINVAL, "buffers overlap");
    for (void *p : {a, b}) {       // both buffers must be device memory with room for `used` bytes
        halos_status st = check_probe_buffer(p, used);
        if (st != HALOS_OK) return st;
    }
    int dev = 0, n_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return fail_hip(e, "querying the device");
    LaunchShape shape;
    shape.grid_cap = g_blocks_per_cu.load() * (n_cu > 0 ? n_cu : 1);
    shape.nontemporal = true;
    hipStream_t s = (hipStream_t)stream;
    float ms = 0.f;
    halos_status st = time_launches(s, reps, [&] { return launch_probe_pair(s, (float *)a, (float *)b, (uint32_t)n_tiles64, shape); }, &ms);
    if (st != HALOS_OK) return st;
    *gbps = ms > 0.f ? (double)used * 4.0 * reps / ((double)ms * 1e-3) / 1e9 : 0.0;
    return HALOS_OK;
}

halos_status halos_probe_streams(const void *const *read_bufs, int32_t n_read, void *const *write_bufs, int32_t n_write,
                                 uint64_t bytes, int32_t reps, int32_t unroll, void *stream, double *gbps) {
    if (!gbps) return fail(HALOS_EINVAL, "gbps is NULL");
    if (unroll == 0) unroll = UNROLL;
    if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8 && unroll != 16)
        return fail(HALOS_EINVAL, "unroll = %d, must be 0 (the update kernels' own), 1, 2, 4, 8 or 16", unroll);
    if (n_read < 0 || n_read > MAX_PROBE_STREAMS || n_write < 0 || n_write > MAX_PROBE_STREAMS || n_read + n_write == 0)
        return fail(HALOS_EINVAL, "n_read = %d, n_write = %d: each 0..%d, not both 0", n_read, n_write, MAX_PROBE_STREAMS);
    if ((n_read > 0 && !read_bufs) || (n_write > 0 && !write_bufs)) return fail(HALOS_EINVAL, "NULL pointer array");
    const uint64_t tile_bytes = (uint64_t)probe_tile_elems(unroll) * sizeof(float);
    if (bytes < tile_bytes) return fail(HALOS_EINVAL, "bytes = %llu, must be >= %llu", (unsigned long long)bytes,
                                        (unsigned long long)tile_bytes);
    if (reps < 1 || reps > 1000) return fail(HALOS_EINVAL, "reps = %d outside 1..1000", reps);
    const uint64_t n_tiles64 = bytes / tile_bytes;
    if (n_tiles64 > 0xFFFFFFFFull) return fail(HALOS_EINVAL, "bytes too large");
    const uint64_t used = n_tiles64 * tile_bytes;
    ProbeArgs args{};
    for (int i = 0; i < n_read; ++i) {
        halos_status st = check_probe_buffer(read_bufs[i], used);
        if (st != HALOS_OK) return st;
        args.rd[i] = (const float *)read_bufs[i];
    }
    for (int i = 0; i < n_write; ++i) {
        halos_status st = check_probe_buffer(write_bufs[i], used);
        if (st != HALOS_OK) return st;
        args.wr[i] = (float *)write_bufs[i];
        const uintptr_t w0 = reinterpret_cast<uintptr_t>(write_bufs[i]);     // a written buffer overlaps nothing else
        for (int j = 0; j < n_read; ++j) {
            const uintptr_t r0 = reinterpret_cast<uintptr_t>(read_bufs[j]);
            if (w0 < r0 + used && r0 < w0 + used) return fail(HALOS_EINVAL, "write buffer %d overlaps read buffer %d", i, j);
        }
        for (int j = 0; j < i; ++j) {
            const uintptr_t o0 = reinterpret_cast<uintptr_t>(write_bufs[j]);
            if (w0 < o0 + used && o0 < w0 + used) return fail(HALOS_EINVAL, "write buffers %d and %d overlap", i, j);
        }
    }
    int dev = 0, n_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return fail_hip(e, "querying the device");
    LaunchShape shape;
    shape.grid_cap = g_blocks_per_cu.load() * (n_cu > 0 ? n_cu : 1);
    shape.nontemporal = true;
    hipStream_t s = (hipStream_t)stream;
    float ms = 0.f;
    halos_status st = time_launches(s, reps, [&] { return launch_probe_streams(s, args, n_read, n_write, unroll, (uint32_t)n_tiles64, shape); }, &ms);
    if (st != HALOS_OK) return st;
    *gbps = ms > 0.f ? (double)used * (n_read + n_write) * reps / ((double)ms * 1e-3) / 1e9 : 0.0;
    return HALOS_OK;
}

halos_status halos_gps_create(const halos_layout *layout, const halos_hparams *hp, void *const *Theta, void *const *M,
                              void *stream, halos_gps **out) {
    if (!out) return fail(HALOS_EINVAL, "out is NULL");
    *out = nullptr;
    if (!layout || !layout->numel) return fail(HALOS_EINVAL, "layout is NULL");
    if (layout->n_tensors < 1) return fail(HALOS_EINVAL, "n_tensors = %d, must be >= 1", layout->n_tensors);
    halos_status st = check_hparams(hp);
    if (st != HALOS_OK) return st;
    for (int32_t i = 0; i < layout->n_tensors; ++i) {
        if (layout->numel[i] < 0) return fail(HALOS_EINVAL, "numel[%d] is negative", i);
        if (layout->numel[i] > (int64_t)0xFFFFFFFFll) return fail(HALOS_EINVAL, "numel[%d] exceeds 2^32-1", i);
    }
    halos_gps *g = new (std::nothrow) halos_gps;
    if (!g) return fail(HALOS_ENOMEM, "host allocation failed");
    hipError_t e = hipGetDevice(&g->device);
    if (e != hipSuccess) { delete g; return fail_hip(e, "hipGetDevice"); }
    int n_cu = 0;
    e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, g->device);
    if (e != hipSuccess) { delete g; return fail_hip(e, "hipDeviceGetAttribute"); }
    g->n_cu = n_cu > 0 ? n_cu : 1;
    g->numel.assign(layout->numel, layout->numel + layout->n_tensors);
    for (int64_t v : g->numel) g->total += v;
    g->hp = *hp;
    g->rule = hp->global;

    g->no_momentum = (hp->flags & HALOS_FLAG_GPS_NO_MOMENTUM) != 0;
    g->momentum_bf16 = (hp->flags & HALOS_FLAG_BF16_MOMENTUM) != 0;
    st = check_tensors(g, Theta, sizeof(float), "Theta");
    if (st == HALOS_OK && !g->no_momentum) st = check_tensors(g, M, g->momentum_bf16 ? 2 : sizeof(float), "M");
    if (st != HALOS_OK) { delete g; return st; }

    // tile table and launch ranges
    std::vector<Tile> tiles;
    const size_t nt = g->numel.size();
    for (size_t base = 0; base < nt; base += MAX_ARG_TENSORS) {
        TileRange r;
        r.tensor_base = (uint32_t)base;
        r.lo = (uint32_t)tiles.size();
        for (size_t t = base; t < nt && t < base + MAX_ARG_TENSORS; ++t)
            for (int64_t s = 0; s < g->numel[t]; s += TILE_ELEMS) {
                Tile tl;
                tl.tensor = (uint32_t)t;
                tl.start = (uint64_t)s;
                tl.len = (uint32_t)((g->numel[t] - s) < TILE_ELEMS ? (g->numel[t] - s) : TILE_ELEMS);
                tiles.push_back(tl);
            }
        r.hi = (uint32_t)tiles.size();
        if (r.hi > r.lo) g->ranges.push_back(r);
    }
    g->n_tiles = (uint32_t)tiles.size();
    e = hipMalloc((void **)&g->d_tiles, tiles.empty() ? sizeof(Tile) : tiles.size() * sizeof(Tile));
    if (e != hipSuccess) { (void)hipGetLastError(); delete g; return fail(HALOS_ENOMEM, "tile table: %s", hipGetErrorString(e)); }
    if (!tiles.empty()) {
        e = hipMemcpy(g->d_tiles, tiles.data(), tiles.size() * sizeof(Tile), hipMemcpyHostToDevice);
        if (e != hipSuccess) { (void)hipFree(g->d_tiles); delete g; return fail_hip(e, "uploading the tile table"); }
    }
    const std::vector<const void *> no_M(nt, nullptr);
    st = upload_tables(&g->d_tables, {(const void *const *)Theta, g->no_momentum ? no_M.data() : (const void *const *)M}, nt, 1);
    if (st != HALOS_OK) { (void)hipFree(g->d_tiles); delete g; return st; }
    g->d_Theta = (float **)g->d_tables;
    g->d_M = g->d_Theta + nt;
    g->d_buffer = g->d_M + nt;

    for (const TileRange &r : g->ranges) {       // M <- 0
        if (g->no_momentum) break;
        e = launch_init((hipStream_t)stream, g->d_tiles, r, nullptr, nullptr, g->d_M, nullptr, false, current_shape(g),
                        g->momentum_bf16);
        if (e != hipSuccess) {
            (void)hipFree(g->d_tables); (void)hipFree(g->d_tiles); delete g;
            return fail_hip(e, "zero-filling M");
        }
    }
    register_handle(g);
    *out = g;
    return HALOS_OK;
}

static void gps_release(halos_gps *g) {
    unregister_handle(g);
    (void)hipFree(g->d_tables);
    (void)hipFree(g->d_tiles);
    g->magic = 0;
    delete g;
}

void halos_gps_destroy(halos_gps *g) {
    if (!live_gps(g)) return;
    if (g->n_lps_attached > 0) {        // its local servers still launch with the layout tables: keep them until the last one goes
        g->retired = true;
        return;
    }
    gps_release(g);
}

halos_status halos_lps_create(halos_gps *g, int32_t lps_id, int32_t n_workers, void *const *theta, void *const *m,
                              void *const *acc, void *stream, halos_lps **out) {
    if (!out) return fail(HALOS_EINVAL, "out is NULL");
    *out = nullptr;
    if (!live_gps(g)) return fail(HALOS_EINVAL, "gps is not a valid handle");
    if (lps_id < 0) return fail(HALOS_EINVAL, "lps_id = %d, must be >= 0", lps_id);
    if (n_workers < 1) return fail(HALOS_EINVAL, "n_workers = %d, must be >= 1", n_workers);
    halos_status st = check_device(g);
    if (st == HALOS_OK) st = check_tensors(g, theta, sizeof(float), "theta");
    if (st == HALOS_OK) st = check_tensors(g, m, g->momentum_bf16 ? 2 : sizeof(float), "m");
    if (st == HALOS_OK) st = check_tensors(g, acc, sizeof(float), "acc");
    if (st != HALOS_OK) return st;
    halos_lps *l = new (std::nothrow) halos_lps(n_workers, g->hp.K);
    if (!l) return fail(HALOS_ENOMEM, "host allocation failed");
    l->gps = g;
    l->id = lps_id;
    l->snapshot = (g->hp.flags & HALOS_FLAG_SNAPSHOT) != 0;
    l->defer_clear = (g->hp.flags & HALOS_FLAG_DEFER_CLEAR) != 0;
    l->rule = g->hp.local;
    l->alpha = g->hp.alpha;
    l->pending.resize(n_workers);
    l->validated.resize(n_workers);
    l->validated_dtype.assign(n_workers, HALOS_F32);
    const size_t nt = g->numel.size();
    st = upload_tables(&l->d_tables, {(const void *const *)theta, (const void *const *)m, (const void *const *)acc}, nt,
                       2 * (size_t)n_workers + 1);
    if (st != HALOS_OK) { delete l; return st; }
    l->d_theta = (float **)l->d_tables;
    l->d_m = l->d_theta + nt;
    l->d_acc = l->d_m + nt;
    l->d_worker_model = l->d_acc + nt;
    l->d_buffer = l->d_worker_model + (size_t)n_workers * nt;
    l->d_delta = l->d_buffer + nt;
    l->delta_in_table.resize(n_workers);
    l->worker_has_model.assign(n_workers, 0);
    l->worker_model_host.resize(n_workers);
    if (g->hp.flags & HALOS_FLAG_NORMS) {
        l->norm_partial_cap = (uint32_t)(g->ranges.size() ? g->ranges.size() : 1) * 64u * (uint32_t)g->n_cu;
        const size_t bytes = ((size_t)l->norm_partial_cap + 2) * sizeof(double);
        hipError_t e = hipMalloc((void **)&l->d_norm_partials, bytes);
        if (e == hipSuccess) e = hipMemset(l->d_norm_partials, 0, bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            if (l->d_norm_partials) (void)hipFree(l->d_norm_partials);
            (void)hipFree(l->d_tables);
            delete l;
            return fail(HALOS_ENOMEM, "norm scratch: %s", hipGetErrorString(e));
        }
        l->d_norm_results = l->d_norm_partials + l->norm_partial_cap;
    }
    for (const TileRange &r : g->ranges) {       // theta <- Theta, m <- 0, acc <- 0
        hipError_t e = launch_init((hipStream_t)stream, g->d_tiles, r, g->d_Theta, l->d_theta, l->d_m, l->d_acc,
                                   l->snapshot, current_shape(g), g->momentum_bf16);
        if (e != hipSuccess) {
            if (l->d_norm_partials) (void)hipFree(l->d_norm_partials);
            (void)hipFree(l->d_tables);
            delete l;
            return fail_hip(e, "initialising the local server");
        }
    }
    g->n_lps_attached += 1;
    register_handle(l);
    *out = l;
    return HALOS_OK;
}

void halos_lps_destroy(halos_lps *l) {
    if (!live_lps(l)) return;
    (void)hipFree(l->d_tables);
    if (l->d_norm_partials) (void)hipFree(l->d_norm_partials);
    halos_gps *g = l->gps;
    unregister_handle(l);
    l->magic = 0;
    delete l;
    if (is_registered(g) && g->magic == GPS_MAGIC) {
        g->n_lps_attached -= 1;
        if (g->retired && g->n_lps_attached == 0) gps_release(g);
    }
}

static halos_status push_delta_impl(halos_lps *l, int32_t worker, const void *const *gptrs, halos_dtype dtype,
                                    uint32_t staleness, bool end_model, float weight) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (dtype != HALOS_F32 && dtype != HALOS_BF16 && dtype != HALOS_F16) return fail(HALOS_EINVAL, "unknown delta dtype %d", (int)dtype);
    if (!std::isfinite(weight)) return fail(HALOS_EINVAL, "weight is not finite");
    ProtoResult pr = l->proto.can_push_delta(worker);
    if (pr == PROTO_BAD_ARG) return fail(HALOS_EINVAL, "worker %d outside 0..%d", worker, l->proto.n_workers() - 1);
    if (pr == PROTO_BAD_STATE) return fail(HALOS_ESTATE, "worker %d of lps %d already has a delta queued", worker, l->id);
    if (end_model && !l->worker_has_model[worker])
        return fail(HALOS_ESTATE, "worker %d of lps %d has no model buffer registered: its start model is unknown", worker, l->id);
    const char *what = end_model ? "end_model" : "g";
    if (!gptrs) return fail(HALOS_EINVAL, "%s: pointer array is NULL", what);
    const halos_gps *g = l->gps;
    const size_t nt = g->numel.size();
    if (end_model) {        // the end model must not be (or overlap) the buffer that holds the start model: g would be 0 or garbage
        const std::vector<const void *> &start = l->worker_model_host[worker];
        for (size_t i = 0; i < nt && i < start.size(); ++i) {
            const uintptr_t a = reinterpret_cast<uintptr_t>(gptrs[i]), b = reinterpret_cast<uintptr_t>(start[i]);
            const uintptr_t len = (uintptr_t)g->numel[i] * sizeof(float);
            if (len && a < b + len && b < a + len)
                return fail(HALOS_EINVAL, "end_model: tensor %zu overlaps the worker's registered model buffer (its start model)", i);
        }
    }
    std::vector<const void *> &seen = l->validated[worker];
    const bool same = seen.size() == nt && l->validated_dtype[worker] == dtype &&
                      std::memcmp(seen.data(), gptrs, nt * sizeof(void *)) == 0;
    if (!same) {      // a worker normally reuses its receive buffers: their ranges are checked once
        halos_status st = check_device(g);
        if (st == HALOS_OK) st = check_tensors(g, gptrs, dtype == HALOS_F32 ? 4 : 2, what);
        if (st != HALOS_OK) return st;
        seen.assign(gptrs, gptrs + nt);
        l->validated_dtype[worker] = dtype;
    }
    PendingDelta &p = l->pending[worker];
    p.ptrs.assign(gptrs, gptrs + nt);
    p.dtype = dtype;
    p.end_model = end_model;
    p.staleness = staleness;
    p.weight = weight;
    if (staleness > l->max_staleness) l->max_staleness = staleness;
    l->proto.push_delta(worker);
    return HALOS_OK;
}

halos_status halos_lps_push_update(halos_lps *l, int32_t worker, const void *const *gptrs, halos_dtype dtype,
                                   uint32_t staleness) {
    return push_delta_impl(l, worker, gptrs, dtype, staleness, false, 1.0f);
}

halos_status halos_lps_push_update_weighted(halos_lps *l, int32_t worker, const void *const *gptrs, halos_dtype dtype,
                                            uint32_t staleness, float weight) {
    return push_delta_impl(l, worker, gptrs, dtype, staleness, false, weight);
}

halos_status halos_lps_push_end_model(halos_lps *l, int32_t worker, const void *const *end_model, uint32_t staleness) {
    return push_delta_impl(l, worker, end_model, HALOS_F32, staleness, true, 1.0f);
}

halos_status halos_lps_push_global(halos_lps *l) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (l->proto.can_push_global() != PROTO_OK)
        return fail(HALOS_ESTATE, "lps %d: no global model is on its way back (phase %d)", l->id, l->proto.phase());
    l->proto.push_global();
    return HALOS_OK;
}

// Rewrite one pointer table of n_tensors entries in stream order (the entries travel in kernel-argument blocks).
static halos_status store_table(hipStream_t stream, float **d_table, const void *const *host_ptrs, size_t n_tensors) {
    for (size_t base = 0; base < n_tensors; base += MAX_ARG_TENSORS) {
        PtrArgs args;
        const size_t count = n_tensors - base < (size_t)MAX_ARG_TENSORS ? n_tensors - base : (size_t)MAX_ARG_TENSORS;
        for (size_t i = 0; i < (size_t)MAX_ARG_TENSORS; ++i) args.p[i] = i < count ? host_ptrs[base + i] : nullptr;
        hipError_t e = launch_store_pointers(stream, d_table, args, (uint32_t)base, (uint32_t)count);
        if (e != hipSuccess) return fail_hip(e, "rewriting a pointer table");
    }
    return HALOS_OK;
}

halos_status halos_lps_set_worker_model(halos_lps *l, int32_t worker, void *const *model, void *stream) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (worker < 0 || worker >= l->proto.n_workers())
        return fail(HALOS_EINVAL, "worker %d outside 0..%d", worker, l->proto.n_workers() - 1);
    const halos_gps *g = l->gps;
    halos_status st = check_device(g);
    if (st == HALOS_OK) st = check_tensors(g, (const void *const *)model, sizeof(float), "model");
    if (st != HALOS_OK) return st;
    const size_t nt = g->numel.size();
    // in stream order: launches already issued on the stream keep the old table, later ones see the new
    st = store_table((hipStream_t)stream, l->d_worker_model + (size_t)worker * nt, (const void *const *)model, nt);
    if (st != HALOS_OK) return st;
    l->worker_has_model[worker] = 1;
    l->worker_model_host[worker].assign((const void *const *)model, (const void *const *)model + nt);
    return HALOS_OK;
}

// ext_partials / ext_results: where the norm monitors of this step go instead of the server's own scratch (both null:
// the server's own, if it has one).
static halos_status lps_step_impl(halos_lps *l, void *stream, halos_step_info *info, bool pull,
                                  double *ext_partials = nullptr, double *ext_results = nullptr) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    halos_gps *g = l->gps;
    double *const norm_partials = ext_partials ? ext_partials : l->d_norm_partials;
    double *const norm_results = ext_partials ? ext_results : l->d_norm_results;
    halos_step_info out{};
    out.worker = -1;
    const QueueItem head = l->proto.head();
    if (head.kind == ITEM_NONE) {
        out.t = l->proto.t();
        out.t_last = l->proto.t_last();
        if (info) *info = out;
        return HALOS_OK;
    }
    halos_status st = check_device(g);
    if (st != HALOS_OK) return st;
    const LaunchShape shape = current_shape(g);
    if (head.kind == ITEM_DELTA) {
        const UpdateOutcome oc = l->proto.preview_update();
        const PendingDelta &p = l->pending[head.worker];
        float *const *pull_tab = nullptr;
        if (p.end_model && !pull)
            return fail(HALOS_ESTATE, "lps %d: worker %d sent its end model; halos_lps_step_pull applies it (the pass "
                        "that reads the worker's start model also replaces it)", l->id, head.worker);
        const int g_kind = p.end_model ? GRAD_END_MODEL
                         : (p.dtype == HALOS_BF16 ? GRAD_BF16 : (p.dtype == HALOS_F16 ? GRAD_F16 : GRAD_F32));
        if (pull) {
            if (!l->worker_has_model[head.worker])
                return fail(HALOS_ESTATE, "worker %d of lps %d has no model buffer registered", head.worker, l->id);
            pull_tab = l->d_worker_model + (size_t)head.worker * g->numel.size();
        }
        // what this update does to the third buffer: add its step (running accumulation), or nothing (an accumulated
        // update is in flight, or the buffer holds the snapshot), or -- snapshot form, accumulation complete --
        // turn the snapshot into theta_{t_last} - theta_t
        // (or, after a merge that did not clear the buffer, restart the accumulation from this update's step)
        const int third_mode = l->snapshot ? (oc.freezes ? THIRD_FREEZE_SNAPSHOT : THIRD_NONE)
                             : (oc.accumulate ? (l->third_stale ? THIRD_RESTART : THIRD_ADD) : THIRD_NONE);
        uint32_t n_partials = 0;
        for (const TileRange &r : g->ranges) {
            PtrArgs args;
            fill_args(args, p.ptrs.data(), r, g->numel.size());
            double *partials = norm_partials ? norm_partials + n_partials : nullptr;
            hipError_t e;
            if (l->cycle.d() > 1) {
                const float inv_d = 1.0f / (float)l->cycle.d();
                e = launch_lps_update_delayed((hipStream_t)stream, g->d_tiles, r, l->d_theta, l->d_m, l->d_buffer, l->d_acc,
                                              pull_tab, args, g_kind, third_mode, (int)l->cycle.next(),
                                              l->rule.eta, l->rule.beta, l->rule.cg * inv_d, inv_d, p.weight, partials, shape);
            } else {
                e = launch_lps_update((hipStream_t)stream, g->d_tiles, r, l->d_theta, l->d_m, l->d_acc, pull_tab, args,
                                      g_kind, third_mode, l->rule.eta, l->rule.beta, l->rule.cg, p.weight, partials, shape,
                                      g->momentum_bf16);
            }
            if (e != hipSuccess) return fail_hip(e, "launching the local update");
            n_partials += launch_grid_size(r, shape);
        }
        if (norm_partials) {
            hipError_t e = launch_norm_finalize((hipStream_t)stream, norm_partials, n_partials, norm_results + 0);
            if (e != hipSuccess) return fail_hip(e, "launching the norm reduction");
        }
        l->proto.commit_update();
        l->cycle.commit();
        if (third_mode == THIRD_RESTART) l->third_stale = false;
        out.kind = 1;
        out.worker = head.worker;
        out.accumulated = oc.accumulate ? 1 : 0;
        out.delta_ready = oc.freezes ? 1 : 0;
    } else {
        const float keep = 1.0f - l->alpha;
        uint32_t n_partials = 0;
        for (const TileRange &r : g->ranges) {
            double *partials = norm_partials ? norm_partials + n_partials : nullptr;
            hipError_t e = launch_lps_merge((hipStream_t)stream, g->d_tiles, r, l->d_theta, l->d_acc, l->alpha, keep,
                                            l->snapshot ? MERGE_SNAPSHOT : (l->defer_clear ? MERGE_LEAVE : MERGE_CLEAR),
                                            partials, shape);
            if (e != hipSuccess) return fail_hip(e, "launching the merge");
            n_partials += launch_grid_size(r, shape);
        }
        if (norm_partials) {
            hipError_t e = launch_norm_finalize((hipStream_t)stream, norm_partials, n_partials, norm_results + 1);
            if (e != hipSuccess) return fail_hip(e, "launching the norm reduction");
        }
        l->proto.commit_merge();
        if (l->defer_clear) l->third_stale = true;
        out.kind = 2;
    }
    out.t = l->proto.t();
    out.t_last = l->proto.t_last();
    if (info) *info = out;
    return HALOS_OK;
}

halos_status halos_lps_step(halos_lps *l, void *stream, halos_step_info *info) {
    return lps_step_impl(l, stream, info, false);
}

halos_status halos_lps_step_pull(halos_lps *l, void *stream, halos_step_info *info) {
    return lps_step_impl(l, stream, info, true);
}

namespace {

// Can the `count` queue items from position `first_item` on go through one multi-delta pass?  All must be plain deltas
// of one element type.
bool multi_eligible(const halos_lps *l, int32_t count, bool pull, int32_t first_item = 0) {
    if (!l->proto.are_deltas(first_item, count)) return false;
    const PendingDelta &first = l->pending[l->proto.item(first_item).worker];
    for (int32_t i = first_item; i < first_item + count; ++i) {
        const int32_t w = l->proto.item(i).worker;
        const PendingDelta &p = l->pending[w];
        if (p.end_model || p.dtype != first.dtype) return false;
        if (pull && !l->worker_has_model[w]) return false;
    }
    return true;
}

// Make worker w's device table of delta pointers hold the pointer set it has queued (rewritten in stream order if it
// holds another), and return the table.
halos_status delta_table(halos_lps *l, int32_t w, hipStream_t stream, const float *const **out) {
    const size_t nt = l->gps->numel.size();
    float **tab = l->d_delta + (size_t)w * nt;
    const PendingDelta &p = l->pending[w];
    std::vector<const void *> &held = l->delta_in_table[w];
    if (held.size() != nt || std::memcmp(held.data(), p.ptrs.data(), nt * sizeof(void *)) != 0) {
        halos_status st = store_table(stream, tab, p.ptrs.data(), nt);
        if (st != HALOS_OK) return st;
        held = p.ptrs;
    }
    *out = tab;
    return HALOS_OK;
}

int grad_kind(halos_dtype d) { return d == HALOS_BF16 ? GRAD_BF16 : (d == HALOS_F16 ? GRAD_F16 : GRAD_F32); }

// Under a momentum delay: the returned global model at the head of the queue and the ONE plain delta behind it, merged
// and applied in one pass (the caller has checked that this is what the queue holds and that the sender has a model
// buffer).  Same results as halos_lps_step followed by halos_lps_step_pull.
halos_status merge_then_delayed_update(halos_lps *l, void *stream, halos_step_info *infos, int32_t *n_done) {
    halos_gps *g = l->gps;
    halos_status st = check_device(g);
    if (st != HALOS_OK) return st;
    LpsProtocol sim = l->proto;
    sim.commit_merge();
    halos_step_info out[2];
    out[0] = halos_step_info{};
    out[0].kind = 2;
    out[0].worker = -1;
    out[0].t = sim.t();
    out[0].t_last = sim.t_last();
    const int32_t w = sim.head().worker;
    const UpdateOutcome oc = sim.preview_update();          // right after a merge every update accumulates
    sim.commit_update();
    const PendingDelta &p = l->pending[w];
    const int third_mode = l->snapshot ? (oc.freezes ? THIRD_FREEZE_SNAPSHOT : THIRD_MERGED_SNAPSHOT) : THIRD_ADD;
    const float inv_d = 1.0f / (float)l->cycle.d();
    const LaunchShape shape = current_shape(g);
    const size_t nt = g->numel.size();
    for (const TileRange &r : g->ranges) {
        PtrArgs args;
        fill_args(args, p.ptrs.data(), r, nt);
        hipError_t e = launch_lps_update_delayed((hipStream_t)stream, g->d_tiles, r, l->d_theta, l->d_m, l->d_buffer, l->d_acc,
                                                 l->d_worker_model + (size_t)w * nt, args, grad_kind(p.dtype), third_mode,
                                                 (int)l->cycle.next(), l->rule.eta, l->rule.beta, l->rule.cg * inv_d, inv_d,
                                                 p.weight, nullptr, shape, true, l->alpha, 1.0f - l->alpha);
        if (e != hipSuccess) return fail_hip(e, "launching the merge and delayed update");
    }
    l->proto = sim;
    l->cycle.commit();
    l->third_stale = false;
    out[1] = halos_step_info{};
    out[1].kind = 1;
    out[1].worker = w;
    out[1].accumulated = oc.accumulate ? 1 : 0;
    out[1].delta_ready = oc.freezes ? 1 : 0;
    out[1].t = l->proto.t();
    out[1].t_last = l->proto.t_last();
    infos[0] = out[0];
    infos[1] = out[1];
    *n_done = 2;
    return HALOS_OK;
}

}  // namespace

halos_status halos_lps_step_average(halos_lps *l, int32_t count, void *stream, halos_step_info *info) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (count < 1 || count > MAX_MULTI) return fail(HALOS_EINVAL, "count = %d outside 1..%d", count, MAX_MULTI);
    halos_gps *g = l->gps;
    if (l->cycle.d() > 1) return fail(HALOS_ESTATE, "lps %d: the averaged step is not available under a momentum delay", l->id);
    if (l->d_norm_partials) return fail(HALOS_ESTATE, "lps %d: the averaged step does not feed the norm monitors", l->id);
    if (!multi_eligible(l, count, false))
        return fail(HALOS_ESTATE, "lps %d: the first %d queue items are not %d worker deltas of one element type", l->id, count, count);
    halos_status st = check_device(g);
    if (st != HALOS_OK) return st;
    const UpdateOutcome oc = l->proto.preview_update();
    MultiArgs a{};
    a.n_in = count;
    a.n_acc = oc.accumulate ? 1 : 0;
    halos_dtype dtype = HALOS_F32;
    int32_t last_worker = -1;
    for (int32_t i = 0; i < count; ++i) {
        const int32_t w = l->proto.item(i).worker;
        st = delta_table(l, w, (hipStream_t)stream, &a.delta[i]);
        if (st != HALOS_OK) return st;
        a.w[i] = l->pending[w].weight;
        dtype = l->pending[w].dtype;
        last_worker = w;
    }
    const int third_mode = l->snapshot ? (oc.freezes ? THIRD_FREEZE_SNAPSHOT : THIRD_NONE)
                         : (oc.accumulate ? (l->third_stale ? THIRD_RESTART : THIRD_ADD) : THIRD_NONE);
    const LaunchShape shape = current_shape(g);
    const float inv_n = 1.0f / (float)count;
    for (const TileRange &r : g->ranges) {
        hipError_t e = launch_lps_update_multi((hipStream_t)stream, g->d_tiles, r, l->d_theta, l->d_m, l->d_acc, a, true,
                                               grad_kind(dtype), third_mode, l->rule.eta, l->rule.beta, l->rule.cg, inv_n, shape,
                                               g->momentum_bf16);
        if (e != hipSuccess) return fail_hip(e, "launching the averaged update");
    }
    l->proto.commit_average(count);
    if (third_mode == THIRD_RESTART) l->third_stale = false;
    if (info) {
        halos_step_info out{};
        out.kind = 1;
        out.worker = last_worker;
        out.accumulated = oc.accumulate ? 1 : 0;
        out.delta_ready = oc.freezes ? 1 : 0;
        out.t = l->proto.t();
        out.t_last = l->proto.t_last();
        *info = out;
    }
    return HALOS_OK;
}

halos_status halos_lps_step_batch(halos_lps *l, int32_t max_items, int32_t pull, void *stream, halos_step_info *infos,
                                  int32_t *n_done) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (max_items < 1 || max_items > MAX_MULTI) return fail(HALOS_EINVAL, "max_items = %d outside 1..%d", max_items, MAX_MULTI);
    if (!infos || !n_done) return fail(HALOS_EINVAL, "infos / n_done is NULL");
    *n_done = 0;
    halos_gps *g = l->gps;
    // the longest run of plain deltas of one element type at the head of the queue, or right behind a returned global
    // model at the head (then the merge opens the pass)
    const int32_t lead = l->proto.head().kind == ITEM_GLOBAL ? 1 : 0;
    if (lead && l->cycle.d() > 1 && !l->d_norm_partials && pull && max_items >= 2 && multi_eligible(l, 1, true, 1))
        return merge_then_delayed_update(l, stream, infos, n_done);
    int32_t count = 0;
    if (l->cycle.d() == 1 && !l->d_norm_partials)
        for (int32_t c = std::min<int32_t>(max_items, l->proto.queued()) - lead; c >= 2 - lead && c >= 1 && count == 0; --c)
            if (multi_eligible(l, c, pull != 0, lead)) count = c;
    if (count < 2 - lead) {             // nothing to batch: one ordinary step
        const QueueItem head = l->proto.head();
        halos_status st = lps_step_impl(l, stream, &infos[0], pull != 0 && head.kind == ITEM_DELTA);
        if (st == HALOS_OK && infos[0].kind != 0) *n_done = 1;
        return st;
    }
    halos_status st = check_device(g);
    if (st != HALOS_OK) return st;
    // what each of the items will mean for the accumulated update, on a copy of the protocol state
    LpsProtocol sim = l->proto;
    MultiArgs a{};
    a.n_in = count;
    halos_step_info out[MAX_MULTI + 1];
    if (lead) {                         // the merge branch of the LPS block, on the copy
        sim.commit_merge();
        out[0] = halos_step_info{};
        out[0].kind = 2;
        out[0].worker = -1;
        out[0].t = sim.t();
        out[0].t_last = sim.t_last();
        a.merge = 1;
        a.alpha = l->alpha;
        a.keep = 1.0f - l->alpha;
    }
    int32_t n_acc = 0, freeze_at = 0;
    halos_dtype dtype = HALOS_F32;
    const size_t nt = g->numel.size();
    for (int32_t i = 0; i < count; ++i) {
        const int32_t w = sim.head().worker;
        const UpdateOutcome oc = sim.preview_update();
        sim.commit_update();
        if (oc.accumulate) n_acc = i + 1;
        if (oc.freezes) freeze_at = i + 1;
        st = delta_table(l, w, (hipStream_t)stream, &a.delta[i]);
        if (st != HALOS_OK) return st;
        a.pull[i] = pull ? l->d_worker_model + (size_t)w * nt : nullptr;
        a.w[i] = l->pending[w].weight;
        dtype = l->pending[w].dtype;
        halos_step_info &o = out[lead + i];
        o = halos_step_info{};
        o.kind = 1;
        o.worker = w;
        o.accumulated = oc.accumulate ? 1 : 0;
        o.delta_ready = oc.freezes ? 1 : 0;
        o.t = sim.t();
        o.t_last = sim.t_last();
    }
    int third_mode;
    if (l->snapshot) { third_mode = (freeze_at || lead) ? THIRD_FREEZE_SNAPSHOT : THIRD_NONE; a.n_acc = freeze_at; }
    else if (lead) { third_mode = THIRD_ADD; a.n_acc = n_acc; }       // the pass itself restarts the accumulation from zero
    else { third_mode = n_acc ? (l->third_stale ? THIRD_RESTART : THIRD_ADD) : THIRD_NONE; a.n_acc = n_acc; }
    const LaunchShape shape = current_shape(g);
    for (const TileRange &r : g->ranges) {
        hipError_t e = launch_lps_update_multi((hipStream_t)stream, g->d_tiles, r, l->d_theta, l->d_m, l->d_acc, a, false,
                                               grad_kind(dtype), third_mode, l->rule.eta, l->rule.beta, l->rule.cg, 1.0f, shape,
                                               g->momentum_bf16);
        if (e != hipSuccess) return fail_hip(e, "launching the batched update");
    }
    l->proto = sim;
    if (third_mode == THIRD_RESTART || lead) l->third_stale = false;
    for (int32_t i = 0; i < lead + count; ++i) infos[i] = out[i];
    *n_done = lead + count;
    return HALOS_OK;
}

halos_status halos_lps_step_norms(halos_lps *l, void *stream, halos_step_info *info, double *norms_out) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (!norms_out) return fail(HALOS_EINVAL, "norms_out is NULL");
    if ((reinterpret_cast<uintptr_t>(norms_out) & 7u) != 0) return fail(HALOS_EINVAL, "norms_out is not 8-byte aligned");
    const halos_gps *g = l->gps;
    halos_status st = check_device(g);
    if (st != HALOS_OK) return st;
    if (l->validated_norm_out != norms_out) {
        hipPointerAttribute_t attr;
        hipError_t e = hipPointerGetAttributes(&attr, norms_out);
        if (e != hipSuccess || (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged)) {
            (void)hipGetLastError();
            return fail(HALOS_EINVAL, "norms_out is not a device pointer");
        }
        hipDeviceptr_t base = nullptr;
        size_t size = 0;
        e = hipMemGetAddressRange(&base, &size, norms_out);
        if (e != hipSuccess) { (void)hipGetLastError(); return fail(HALOS_EINVAL, "norms_out: cannot query its allocation"); }
        if (reinterpret_cast<uintptr_t>(norms_out) + 2 * sizeof(double) > reinterpret_cast<uintptr_t>(base) + size)
            return fail(HALOS_EINVAL, "norms_out has no room for two doubles");
        l->validated_norm_out = norms_out;
    }
    // one partial sum per workgroup of every launch of the step: they must fit the fixed array
    const LaunchShape shape = current_shape(g);
    uint64_t need = 0;
    for (const TileRange &r : g->ranges) need += launch_grid_size(r, shape);
    if (need > STATIC_SCRATCH_DOUBLES)
        return fail(HALOS_EINVAL, "this layout and launch shape need %llu partial sums; the fixed scratch array holds %u "
                    "(lower blocks_per_cu, or use a server created under HALOS_FLAG_NORMS)", (unsigned long long)need,
                    STATIC_SCRATCH_DOUBLES);
    double *partials = nullptr;
    hipError_t e = static_scratch(&partials);
    if (e != hipSuccess) return fail_hip(e, "locating the fixed scratch array");
    return lps_step_impl(l, stream, info, false, partials, norms_out);
}

halos_status halos_gps_merge(halos_gps *g, halos_lps *from, void *stream) {
    if (!live_gps(g)) return fail(HALOS_EINVAL, "gps is not a valid handle");
    if (!live_lps(from)) return fail(HALOS_EINVAL, "from is not a valid handle");
    if (from->gps != g) return fail(HALOS_EINVAL, "lps %d belongs to another global server", from->id);
    if (from->proto.can_consume() != PROTO_OK)
        return fail(HALOS_ESTATE, "lps %d has no accumulated update waiting (phase %d)", from->id, from->proto.phase());
    halos_status st = check_device(g);
    if (st != HALOS_OK) return st;
    const LaunchShape shape = current_shape(g);
    for (const TileRange &r : g->ranges) {
        hipError_t e;
        if (g->cycle.d() > 1) {
            const float inv_d = 1.0f / (float)g->cycle.d();
            e = launch_gps_update_delayed((hipStream_t)stream, g->d_tiles, r, g->d_Theta, g->d_M, g->d_buffer, from->d_acc,
                                          from->d_acc, (int)g->cycle.next(), g->rule.eta, g->rule.beta, g->rule.cg * inv_d,
                                          inv_d, shape);
        } else if (g->no_momentum) {
            e = launch_gps_update_nomom((hipStream_t)stream, g->d_tiles, r, g->d_Theta, from->d_acc, from->d_acc,
                                        g->rule.eta, g->rule.cg, shape);
        } else {
            e = launch_gps_update((hipStream_t)stream, g->d_tiles, r, g->d_Theta, g->d_M, from->d_acc, from->d_acc,
                                  g->rule.eta, g->rule.beta, g->rule.cg, shape, g->momentum_bf16);
        }
        if (e != hipSuccess) return fail_hip(e, "launching the global update");
    }
    g->cycle.commit();
    from->proto.consume();
    g->updates += 1;
    return HALOS_OK;
}

halos_status halos_gps_push_update(halos_gps *g, const void *const *gptrs, halos_dtype dtype, float weight, void *stream) {
    if (!live_gps(g)) return fail(HALOS_EINVAL, "gps is not a valid handle");
    if (dtype != HALOS_F32 && dtype != HALOS_BF16 && dtype != HALOS_F16) return fail(HALOS_EINVAL, "unknown delta dtype %d", (int)dtype);
    if (!std::isfinite(weight)) return fail(HALOS_EINVAL, "weight is not finite");
    if (g->no_momentum)
        return fail(HALOS_ESTATE, "this global server was created without a momentum array (HALOS_FLAG_GPS_NO_MOMENTUM)");
    if (!gptrs) return fail(HALOS_EINVAL, "g: pointer array is NULL");
    halos_status st = check_device(g);
    if (st != HALOS_OK) return st;
    const size_t nt = g->numel.size();
    const bool same = g->validated_delta.size() == nt && g->validated_delta_dtype == dtype &&
                      std::memcmp(g->validated_delta.data(), gptrs, nt * sizeof(void *)) == 0;
    if (!same) {
        st = check_tensors(g, gptrs, dtype == HALOS_F32 ? 4 : 2, "g");
        if (st != HALOS_OK) return st;
        g->validated_delta.assign(gptrs, gptrs + nt);
        g->validated_delta_dtype = dtype;
    }
    const LaunchShape shape = current_shape(g);
    const int g_kind = dtype == HALOS_BF16 ? GRAD_BF16 : (dtype == HALOS_F16 ? GRAD_F16 : GRAD_F32);
    for (const TileRange &r : g->ranges) {
        PtrArgs args;
        fill_args(args, gptrs, r, nt);
        hipError_t e;
        if (g->cycle.d() > 1) {
            const float inv_d = 1.0f / (float)g->cycle.d();
            e = launch_lps_update_delayed((hipStream_t)stream, g->d_tiles, r, g->d_Theta, g->d_M, g->d_buffer, nullptr, nullptr,
                                          args, g_kind, THIRD_NONE, (int)g->cycle.next(), g->rule.eta, g->rule.beta,
                                          g->rule.cg * inv_d, inv_d, weight, nullptr, shape);
        } else {
            e = launch_lps_update((hipStream_t)stream, g->d_tiles, r, g->d_Theta, g->d_M, nullptr, nullptr, args, g_kind,
                                  THIRD_NONE, g->rule.eta, g->rule.beta, g->rule.cg, weight, nullptr, shape, g->momentum_bf16);
        }
        if (e != hipSuccess) return fail_hip(e, "launching the global server's update");
    }
    g->cycle.commit();
    g->updates += 1;
    return HALOS_OK;
}

halos_status halos_pull_model(const void *server, int32_t is_gps, void *const *dst, void *stream) {
    if (!server) return fail(HALOS_EINVAL, "server is NULL");
    const halos_gps *g = nullptr;
    float *const *src = nullptr;
    halos_lps *l = nullptr;
    if (is_gps) {
        g = static_cast<const halos_gps *>(server);
        if (!live_gps(g)) return fail(HALOS_EINVAL, "server is not a valid gps handle");
        src = g->d_Theta;
    } else {
        l = const_cast<halos_lps *>(static_cast<const halos_lps *>(server));
        if (!live_lps(l)) return fail(HALOS_EINVAL, "server is not a valid lps handle");
        g = l->gps;
        src = l->d_theta;
    }
    if (!dst) return fail(HALOS_EINVAL, "dst: pointer array is NULL");
    const size_t nt = g->numel.size();
    const bool same = l && l->validated_pull.size() == nt &&
                      std::memcmp(l->validated_pull.data(), dst, nt * sizeof(void *)) == 0;
    if (!same) {
        halos_status st = check_device(g);
        if (st == HALOS_OK) st = check_tensors(g, (const void *const *)dst, sizeof(float), "dst");
        if (st != HALOS_OK) return st;
        if (l) l->validated_pull.assign((const void *const *)dst, (const void *const *)dst + nt);
    }
    const LaunchShape shape = current_shape(g);
    for (const TileRange &r : g->ranges) {
        PtrArgs args;
        fill_args(args, (const void *const *)dst, r, nt);
        hipError_t e = launch_pull((hipStream_t)stream, g->d_tiles, r, src, args, shape);
        if (e != hipSuccess) return fail_hip(e, "launching the model copy");
    }
    return HALOS_OK;
}

halos_status halos_set_hparams(void *server, int32_t is_gps, const halos_hparams *hp) {
    if (!server) return fail(HALOS_EINVAL, "server is NULL");
    halos_status st = check_hparams(hp);
    if (st != HALOS_OK) return st;
    if (is_gps) {
        halos_gps *g = static_cast<halos_gps *>(server);
        if (!live_gps(g)) return fail(HALOS_EINVAL, "server is not a valid gps handle");
        if (g->no_momentum && hp->global.beta != 0.0f)
            return fail(HALOS_EINVAL, "this global server keeps no momentum (HALOS_FLAG_GPS_NO_MOMENTUM): global.beta must stay 0");
        g->rule = hp->global;
        g->hp.global = hp->global;
    } else {
        halos_lps *l = static_cast<halos_lps *>(server);
        if (!live_lps(l)) return fail(HALOS_EINVAL, "server is not a valid lps handle");
        l->rule = hp->local;
        l->alpha = hp->alpha;
        l->proto.set_K(hp->K);
    }
    return HALOS_OK;
}

halos_status halos_forget_buffers(void *server, int32_t is_gps) {
    if (!server) return fail(HALOS_EINVAL, "server is NULL");
    if (is_gps) {
        halos_gps *g = static_cast<halos_gps *>(server);
        if (!live_gps(g)) return fail(HALOS_EINVAL, "server is not a valid gps handle");
        g->validated_delta.clear();
    } else {
        halos_lps *l = static_cast<halos_lps *>(server);
        if (!live_lps(l)) return fail(HALOS_EINVAL, "server is not a valid lps handle");
        for (auto &v : l->validated) v.clear();
        l->validated_pull.clear();
        l->validated_norm_out = nullptr;
    }
    return HALOS_OK;
}

halos_status halos_lps_set_threshold(halos_lps *l, int32_t K) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (l->proto.set_K(K) != PROTO_OK) return fail(HALOS_EINVAL, "K = %d, must be >= 1", K);
    return HALOS_OK;
}

halos_status halos_lps_get_counters(const halos_lps *l, int64_t *t, int64_t *t_last, int32_t *phase, int32_t *queued,
                                    uint32_t *max_staleness) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (t) *t = l->proto.t();
    if (t_last) *t_last = l->proto.t_last();
    if (phase) *phase = l->proto.phase();
    if (queued) *queued = l->proto.queued();
    if (max_staleness) *max_staleness = l->max_staleness;
    return HALOS_OK;
}

halos_status halos_lps_get_norms(const halos_lps *l, void *stream, double *out) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (!out) return fail(HALOS_EINVAL, "out is NULL");
    if (!l->d_norm_results) return fail(HALOS_ESTATE, "lps %d was created without HALOS_FLAG_NORMS", l->id);
    hipError_t e = hipMemcpyAsync(out, l->d_norm_results, 2 * sizeof(double), hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "reading the norms");
    return HALOS_OK;
}

// Shared by both tiers: check, wait for the device, store the buffer's pointers in the server's table slot.
static halos_status set_momentum_delay(const halos_gps *g, MomentumCycle &cycle, float **d_slot, int32_t d,
                                       void *const *buffer, void *stream, const char *who) {
    if (d < 1) return fail(HALOS_EINVAL, "d = %d, must be >= 1", d);
    if (d > 1 && g->momentum_bf16)
        return fail(HALOS_ESTATE, "%s keeps its momentum in bfloat16 (HALOS_FLAG_BF16_MOMENTUM): the delayed rule is not built for that", who);
    if (cycle.seen() != 0)
        return fail(HALOS_ESTATE, "%s is %d updates into a cycle of %d: the delay can change only between cycles", who,
                    cycle.seen(), cycle.d());
    if (d > 1) {
        halos_status st = check_device(g);
        if (st == HALOS_OK) st = check_tensors(g, (const void *const *)buffer, sizeof(float), "buffer");
        if (st != HALOS_OK) return st;
        st = store_table((hipStream_t)stream, d_slot, (const void *const *)buffer, g->numel.size());
        if (st != HALOS_OK) return st;
    }
    cycle.set_d(d);
    return HALOS_OK;
}

halos_status halos_lps_set_momentum_delay(halos_lps *l, int32_t d, void *const *buffer, void *stream) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    return set_momentum_delay(l->gps, l->cycle, l->d_buffer, d, buffer, stream, "the local server");
}

halos_status halos_gps_set_momentum_delay(halos_gps *g, int32_t d, void *const *buffer, void *stream) {
    if (!live_gps(g)) return fail(HALOS_EINVAL, "gps is not a valid handle");
    if (g->no_momentum && d > 1)
        return fail(HALOS_ESTATE, "this global server keeps no momentum (HALOS_FLAG_GPS_NO_MOMENTUM): nothing to delay");
    return set_momentum_delay(g, g->cycle, g->d_buffer, d, buffer, stream, "the global server");
}

halos_status halos_lps_get_momentum_delay(const halos_lps *l, int32_t *d, int32_t *seen) {
    if (!live_lps(l)) return fail(HALOS_EINVAL, "lps is not a valid handle");
    if (d) *d = l->cycle.d();
    if (seen) *seen = l->cycle.seen();
    return HALOS_OK;
}

halos_status halos_gps_get_momentum_delay(const halos_gps *g, int32_t *d, int32_t *seen) {
    if (!live_gps(g)) return fail(HALOS_EINVAL, "gps is not a valid handle");
    if (d) *d = g->cycle.d();
    if (seen) *seen = g->cycle.seen();
    return HALOS_OK;
}

halos_status halos_gps_get_counters(const halos_gps *g, int64_t *updates) {
    if (!live_gps(g)) return fail(HALOS_EINVAL, "gps is not a valid handle");
    if (updates) *updates = g->updates;
    return HALOS_OK;
}

}  // extern "C"
