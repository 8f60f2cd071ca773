// Launch interface between the C ABI (halos.cpp) and the gfx950 kernels (kernels.hip).
#pragma once

#include <hip/hip_runtime_api.h>

#include <cstdint>

namespace halos {

// Work is cut into tiles: a tile is a run of at most TILE_ELEMS consecutive elements of ONE tensor,
// starting at a multiple of TILE_ELEMS inside it.  The tile table is built once per layout and lives
// in device memory; a persistent grid walks it with a grid stride.
constexpr int BLOCK_THREADS = 256;      // 4 wavefronts of 64
constexpr int VEC = 4;                  // fp32 elements per 128-bit access
#ifndef HALOS_UNROLL
#define HALOS_UNROLL 4                  // compile-time knob, for measuring other tile sizes (2, 8, 16)
#endif
constexpr int UNROLL = HALOS_UNROLL;    // 128-bit accesses per thread per stream and tile
constexpr int TILE_ELEMS = BLOCK_THREADS * VEC * UNROLL;   // 4096

struct Tile {
    uint32_t tensor;    // index into the per-tensor pointer tables
    uint32_t len;       // 1..TILE_ELEMS
    uint64_t start;     // element offset inside the tensor, multiple of TILE_ELEMS
};

// Pointers that change from call to call (a worker's delta tensors, a pull destination) travel in the
// kernel-argument block, so no device table has to be rewritten while earlier launches may still read it.
constexpr int MAX_ARG_TENSORS = 384;
struct PtrArgs {
    const void *p[MAX_ARG_TENSORS];     // p[i] belongs to tensor (tensor_base + i)
};

struct LaunchShape {
    int grid_cap;       // upper bound on workgroups per launch (blocks_per_cu * compute units)
    bool nontemporal;
};

struct TileRange {      // tiles [lo, hi) all belong to tensors [tensor_base, tensor_base + MAX_ARG_TENSORS)
    uint32_t lo, hi;
    uint32_t tensor_base;
};

// Worker-delta step of a local server: m <- beta m + g; s = eta (cg g + beta m); theta <- theta - s;
// The update is applied to gw * g, gw being the caller's scalar on this delta (1 changes nothing).
// third_mode 1: acc <- acc + s (ModelUpdate of App. E fused with the accumulation behind Alg. 1's Delta);
// third_mode 2: the third buffer holds theta_{t_last} and is overwritten with theta_{t_last} - theta_t (Alg. 1's Delta as
// written, sign flipped); third_mode 0: the third buffer is not touched.
// If `pull` is not null it is a device table of destination tensors that also receive the updated theta
// (Alg. 1, "schedule the worker": the model handed back to the worker, written in the same pass).
// If `norm_partials` is not null the launch also leaves, per workgroup, the sum of g^2 over the workgroup's tiles in
// norm_partials[0 .. launch_grid_size(r, shape)).
// g_kind says what the tensors in `g` hold: the pseudo-gradient in fp32 or bf16, or (GRAD_END_MODEL, needs `pull`)
// the worker's END model in fp32 -- the pseudo-gradient is then formed in the kernel as start - end, the start model
// being what `pull` points to before this launch overwrites it (the delta of Alg. 1's worker block formed on the server, sign flipped).
// third_mode 3: the accumulation restarts with this update, acc <- 0 + s, without reading the buffer (used after a merge
// that left the returned model there instead of clearing it).
// GRAD_F16: the tensors in `g` hold IEEE half values (upcast exactly).
constexpr int GRAD_F32 = 0, GRAD_BF16 = 1, GRAD_END_MODEL = 2, GRAD_F16 = 3;
constexpr int THIRD_NONE = 0, THIRD_ADD = 1, THIRD_FREEZE_SNAPSHOT = 2, THIRD_RESTART = 3;
constexpr int THIRD_MERGED_SNAPSHOT = 4;      // merge-first pass in the snapshot form: the third buffer receives the merged model
// m_bf16: the momentum tensors hold bfloat16; every new momentum is rounded to bfloat16 (nearest even) before it enters
// the step and is stored as 16 bits.
hipError_t launch_lps_update(hipStream_t stream, const Tile *tiles, TileRange r, float *const *theta, float *const *m,
                             float *const *acc, float *const *pull, const PtrArgs &g, int g_kind, int third_mode,
                             float eta, float beta, float cg, float gw, double *norm_partials, LaunchShape shape,
                             bool m_bf16 = false);

// Several worker deltas in ONE pass over the server's state.  The deltas are found through device pointer tables (one per
// delta: table[tensor] is that delta's tensor), because several lists of pointers do not fit a kernel-argument block.
//   sequential (average = false): the n_in deltas are applied one after the other, in order, to each element while it
//       is in registers -- the same operations in the same order as n_in single passes, but m, theta and the third
//       buffer are read and written once.  The first n_acc of them count towards the accumulated update (n_acc = 0:
//       none; under third_mode THIRD_FREEZE_SNAPSHOT the n_acc-th completes it).  pull[i], if not null, receives the
//       model right after delta i was applied (that worker's next start model).
//   average (average = true): ONE ModelUpdate with (w_0 g_0 + ... + w_{n-1} g_{n-1}) * inv_n, added in that order;
//       n_acc is 1 if the update counts, 0 if not; pull tables are ignored.
//   merge first (a.merge != 0, sequential only): the third buffer holds the returned global model Theta_i; before
//       the first delta each element is merged, theta <- alpha Theta_i + keep theta (the merge of Alg. 1's LPS block),
//       and the accumulation restarts: the third buffer leaves the pass as the sum of the first n_acc steps
//       (third_mode THIRD_ADD), or, in the snapshot form (THIRD_FREEZE_SNAPSHOT), as the merged model -- turned into
//       theta_{t_last} - theta_t by the n_acc-th update if n_acc > 0.  Same operations in the same order as a merge
//       pass followed by the update passes; the merge pass's 16 bytes per parameter are not moved.
// dtype of all deltas: GRAD_F32, GRAD_BF16 or GRAD_F16.  Always non-temporal; no norm monitors.
constexpr int MAX_MULTI = 4;
struct MultiArgs {
    const float *const *delta[MAX_MULTI];    // device tables of n_tensors pointers each (element type per g_kind)
    float *const *pull[MAX_MULTI];           // device tables, or null
    float w[MAX_MULTI];                      // the callers' scalars on the deltas
    int32_t n_in;                            // 2..MAX_MULTI (1 is allowed)
    int32_t n_acc;
    int32_t merge;                           // 1: merge the returned global model first (see above)
    float alpha, keep;                       // merge weights (used if merge)
};
hipError_t launch_lps_update_multi(hipStream_t stream, const Tile *tiles, TileRange r, float *const *theta, float *const *m,
                                   float *const *acc, const MultiArgs &a, bool average, int g_kind, int third_mode,
                                   float eta, float beta, float cg, float inv_n, LaunchShape shape, bool m_bf16 = false);

// Number of workgroups a launch over range r uses (0 for an empty range).
uint32_t launch_grid_size(TileRange r, LaunchShape shape);

// *out = sum of partials[0..n), added in a fixed order by one workgroup.
hipError_t launch_norm_finalize(hipStream_t stream, const double *partials, uint32_t n, double *out);

// Global-server step: M <- beta M + G; Theta <- Theta - eta (cg G + beta M); out <- Theta.
// `G` and `out` may be the same table (each element is read before it is overwritten by the same thread).
hipError_t launch_gps_update(hipStream_t stream, const Tile *tiles, TileRange r, float *const *Theta, float *const *M,
                             float *const *G, float *const *out, float eta, float beta, float cg, LaunchShape shape,
                             bool m_bf16 = false);

// The global-server step without momentum (beta_g = 0, Sec. 5.4): Theta <- Theta - eta (cg G); out <- Theta.  No
// momentum array is touched.
hipError_t launch_gps_update_nomom(hipStream_t stream, const Tile *tiles, TileRange r, float *const *Theta,
                                   float *const *G, float *const *out, float eta, float cg, LaunchShape shape);

// The same two steps under delayed Nesterov momentum (Sec. 5.1; App. D, delays d_l and d_g).  cycle_pos says where
// in its cycle of d updates the server is: CYCLE_FIRST (buffer <- g), CYCLE_INNER (buffer <- buffer + g) or
// CYCLE_REFRESH (m <- beta m + (buffer + g) * inv_d, then applied; the buffer is left as it is).  Every update
// steps the model by eta * cgd * g (cgd = cg / d); only a refresh reads or writes m.  Always non-temporal.
// norm_partials as in launch_lps_update.
// merge (local server only; needs pull, no monitors, no end model): the third buffer holds the returned global model;
// every element is merged first, theta <- alpha Theta_i + keep theta, and the accumulation restarts with this update
// (third_mode THIRD_ADD: third <- 0 + step; THIRD_FREEZE_SNAPSHOT: third <- merged - updated; THIRD_MERGED_SNAPSHOT:
// third <- merged).  Same operations in the same order as a merge pass followed by the update pass.
constexpr int CYCLE_FIRST = 1, CYCLE_INNER = 2, CYCLE_REFRESH = 3;
hipError_t launch_lps_update_delayed(hipStream_t stream, const Tile *tiles, TileRange r, float *const *theta,
                                     float *const *m, float *const *buffer, float *const *acc, float *const *pull,
                                     const PtrArgs &g, int g_kind, int third_mode, int cycle_pos, float eta,
                                     float beta, float cgd, float inv_d, float gw, double *norm_partials, LaunchShape shape,
                                     bool merge = false, float alpha = 0.f, float keep = 0.f);
hipError_t launch_gps_update_delayed(hipStream_t stream, const Tile *tiles, TileRange r, float *const *Theta,
                                     float *const *M, float *const *buffer, float *const *G, float *const *out,
                                     int cycle_pos, float eta, float beta, float cgd, float inv_d, LaunchShape shape);

// Merge step of a local server: theta <- alpha * inbox + keep * theta (keep = 1 - alpha).
// third_out: what the inbox buffer receives -- MERGE_CLEAR zeros, MERGE_SNAPSHOT the merged model (the new
// theta_{t_last}), MERGE_LEAVE nothing (the next accumulating update must then run with THIRD_RESTART).
// With `norm_partials`: per workgroup, the sum of (theta - inbox)^2 before the merge (same layout as above).
constexpr int MERGE_CLEAR = 0, MERGE_SNAPSHOT = 1, MERGE_LEAVE = 2;
hipError_t launch_lps_merge(hipStream_t stream, const Tile *tiles, TileRange r, float *const *theta,
                            float *const *inbox, float alpha, float keep, int third_out, double *norm_partials,
                            LaunchShape shape);

// table[first + i] <- src.p[i] for i < count (count <= MAX_ARG_TENSORS): rewrites part of a device pointer table in
// stream order, so that launches issued earlier on the stream still see the old entries and later ones the new.
hipError_t launch_store_pointers(hipStream_t stream, float **table, const PtrArgs &src, uint32_t first, uint32_t count);

// Per-workgroup partial sums for callers that may not allocate: a fixed array in the library's device image, one copy
// per GPU, STATIC_SCRATCH_DOUBLES doubles long.  *ptr receives its address on the CURRENT device (looked up once per
// device and remembered).  Whatever an earlier launch left there stays there; launches that use it must not overlap.
constexpr uint32_t STATIC_SCRATCH_DOUBLES = 16384;      // 128 KiB
hipError_t static_scratch(double **ptr);

// dst <- src (fp32), dst pointers in the argument block.
hipError_t launch_pull(hipStream_t stream, const Tile *tiles, TileRange r, float *const *src, const PtrArgs &dst,
                       LaunchShape shape);

// theta <- src; m <- 0; acc <- 0   (Alg. 1, LPS initialisation).  src == nullptr: only zero-fill `m` (used for the GPS momentum).
// `snapshot`: acc <- src instead of 0.
hipError_t launch_init(hipStream_t stream, const Tile *tiles, TileRange r, float *const *src, float *const *theta,
                       float *const *m, float *const *acc, bool snapshot, LaunchShape shape, bool m_bf16 = false);

// Sweep the first n_tiles * TILE_ELEMS floats of two buffers (read both, write both back unchanged).
hipError_t launch_probe_pair(hipStream_t stream, float *a, float *b, uint32_t n_tiles, LaunchShape shape);

// Read n_read buffers and write zeros to n_write others, with the access pattern of the update kernels and no
// arithmetic: what the memory system delivers for that mix of streams.  `unroll` (1, 2, 4, 8 or 16) is the number of
// 128-bit accesses per thread, stream and tile: a probe tile is BLOCK_THREADS * VEC * unroll floats (probe_tile_elems),
// and the first n_tiles of them are swept in every buffer.
constexpr int MAX_PROBE_STREAMS = 4;
struct ProbeArgs {
    const float *rd[MAX_PROBE_STREAMS];
    float *wr[MAX_PROBE_STREAMS];
};
constexpr uint32_t probe_tile_elems(int unroll) { return (uint32_t)(BLOCK_THREADS * VEC * unroll); }
hipError_t launch_probe_streams(hipStream_t stream, const ProbeArgs &a, int n_read, int n_write, int unroll,
                                uint32_t n_tiles, LaunchShape shape);

}  // namespace halos
