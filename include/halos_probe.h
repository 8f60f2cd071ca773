/*
 * halos_probe.h -- measurement and placement helpers of the HALoS update library.
 *
 * These calls are NOT steps of the algorithm: they time plain streaming kernels with the access pattern of the
 * update kernels, so that a caller can sort device memory by HBM region (halos_probe_pair; the arena of
 * include/halos.h is built on it) and see what the memory system delivers to a given mix of read and written
 * streams (halos_probe_streams; the benchmark's ceilings mode).  Same conventions as include/halos.h.
 */
#ifndef HALOS_PROBE_H
#define HALOS_PROBE_H

#include <stdint.h>

#include "halos.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Memory-placement helper (not a step of the algorithm).  An MI355X serves its 288 GB of HBM from a few
 * independent regions, and a kernel whose read-modify-write streams live in different regions gets
 * noticeably more bandwidth than one whose streams share a region.  This call sweeps the two device
 * buffers `reps` times on `stream` (each element is read and written back unchanged), waits for the
 * sweeps, and reports the achieved GB/s (4 x bytes per sweep).  Two buffers in the same region report a
 * visibly lower figure than two buffers in different regions, which lets a caller that allocates its
 * state in slabs sort the slabs by region and put theta, m and acc of a server into different ones.
 *   a, b    16-byte aligned device buffers of at least `bytes` bytes each; must not overlap; no other
 *           work may write them while the call runs
 *   bytes   >= 16 KiB; rounded down to a multiple of 16 KiB
 *   reps    1..1000 timed sweeps (one untimed sweep runs first)
 * Errors: EINVAL, EHIP.
 */
halos_status halos_probe_pair(void *a, void *b, uint64_t bytes, int32_t reps, void *stream, double *gbps);

/*
 * Measurement helper (not a step of the algorithm): what the memory system delivers to a kernel that streams
 * n_read buffers in and n_write other buffers out with the access pattern of the update kernels (tiles of 16 KiB by default,
 * 128-bit non-temporal accesses, all loads of a tile issued first) and no arithmetic.  It gives the ceiling that an
 * update pass with the same mix of read and written streams, placed the same way, can reach on this device.
 *   read_bufs   host array of n_read device buffers, only read
 *   write_bufs  host array of n_write device buffers, OVERWRITTEN WITH ZEROS; none may overlap any other buffer
 *   n_read, n_write   0..4 each, not both 0
 *   bytes, reps, stream   as for halos_probe_pair (every buffer at least `bytes` long, 16-byte aligned); bytes is
 *           rounded down to a multiple of the probe's tile, unroll x 4 KiB
 *   unroll  128-bit accesses per thread, stream and tile: 1, 2, 4, 8 or 16 (tiles of 4 .. 64 KiB), or 0 for the
 *           update kernels' own value; lets a caller see whether longer same-direction bursts would help
 *   gbps        achieved GB/s, counting (n_read + n_write) x bytes per sweep
 * Errors: EINVAL, EHIP.
 */
halos_status halos_probe_streams(const void *const *read_bufs, int32_t n_read, void *const *write_bufs, int32_t n_write,
                                 uint64_t bytes, int32_t reps, int32_t unroll, void *stream, double *gbps);

#ifdef __cplusplus
}
#endif
#endif /* HALOS_PROBE_H */
