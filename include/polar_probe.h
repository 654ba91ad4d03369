/*
 * polar_probe.h — C ABI of the read yardsticks (libpolar_probe.so).
 *
 * Measurement aids for harnesses, kept out of the product library (polar.h): kernels that do
 * nothing but read memory in the access pattern of one of the library's streaming kernels, so a
 * benchmark can set the bandwidth a kernel reaches beside the bandwidth the bare access pattern
 * reaches on the same GPU.  No operation of the paper lives here.  Conventions are those of
 * polar.h: device pointers owned by the caller, no allocation, no synchronisation, kernels are
 * enqueued on `stream` (a hipStream_t as void*, NULL = default stream), the return value is a
 * polar_status, every argument check runs on the host before any HIP call.
 */
#ifndef POLAR_PROBE_H
#define POLAR_PROBE_H

#include <stddef.h>
#include <stdint.h>

#include "polar.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Streaming-read yardstick (not an operation of the paper): `slabs` workgroups
 * each read one contiguous slab of `slab_bytes` bytes (slab w starts at src + w * slab_bytes)
 * with the per-head streaming kernel's launch shape and fold what they read into sink[w].
 * Timing it over the bytes of a K cache gives the read bandwidth this GPU reaches for that
 * access pattern, to set beside the nominal HBM peak.  nontemporal != 0 marks the loads
 * non-temporal, as the attention kernels do.
 *   src  in   slabs * slab_bytes bytes, 16-byte aligned; slab_bytes a multiple of 16
 *   sink out  [slabs] uint32
 */
int polar_probe_read(const void *src, size_t slabs, size_t slab_bytes, int nontemporal, uint32_t *sink,
                     void *stream);

/*
 * The same kind of yardstick for the selective GEMMs (not an operation of the paper): reads the
 * rows W[idx[j], :] (j < n_idx) of a [N, K] 16-bit matrix the way those kernels stream them,
 * in 256-byte pieces, 4 rows per wave-wide load, and does nothing else.  Workgroup (tile, slice) of
 * two waves takes 64 consecutive entries of idx and the slice-th of `slices` equal parts of K;
 * `depth` (1 or 4) 128-value blocks are in flight per wave.  Timing it over n_idx * K * 2 bytes
 * gives the read bandwidth this access pattern reaches by itself.
 *   W     in   [N, K] 16-bit, 16-byte aligned; K a multiple of 128 * slices * depth
 *   idx   in   [n_idx] int32; an id outside [0,N) reads row 0
 *   sink  out  [2 * ceil(n_idx / 64) * slices] uint32
 */
int polar_probe_gather_read(const void *W, const int32_t *idx, int n_idx, int N, int K, int slices, int depth,
                            int nontemporal, uint32_t *sink, void *stream);

/* The hipError_t (as int) recorded by the most recent POLAR_EHIP of this library on this thread; 0 if none. */
int polar_probe_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* POLAR_PROBE_H */
