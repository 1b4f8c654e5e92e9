/*
 * ssd_measure.h - measurement kernels of the SSD build, in a library of their own
 * (libssd_measure.so).  They time the memory system with the access patterns of the
 * weight-streaming GEMM (the dominant kernel of the verification forward, Section 3.2.4,
 * Eq. 5) and are no part of the decoding path: the product library exports none of them.
 * Return 0 or a negative code (-1 invalid argument, -4 HIP error).
 */
#ifndef SSD_MEASURE_H
#define SSD_MEASURE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Streams `bytes` of device memory with the access pattern of the GEMM's weight stream
 * (work_groups x waves_per_wg waves, `depth` 16-byte loads in flight per lane: 4, 8 or 16):
 * the HBM read rate the chip sustains, i.e. the practical ceiling of the roofline.
 * `sink` is 16 bytes of device scratch.  Asynchronous on `hip_stream`. */
int ssd_measure_stream_read(const void* src, size_t bytes, int work_groups, int waves_per_wg, int depth,
                            void* sink, void* hip_stream);

/* The loads of a weight-streaming GEMM and nothing else: each of `work_groups` work-groups
 * reads all shared_bytes of `shared` (the activations every work-group needs) and its own
 * priv_bytes_per_wg of `priv` (work-group g reads [g, g+1) * priv_bytes_per_wg: its share of the
 * weights, non-temporal), evenly interleaved, with `threads` (512 or 1024) lanes and `depth` (4 or 8)
 * 16-byte loads in flight per lane.  Both sizes must be multiples of threads * depth * 16 bytes; `priv`
 * must hold work_groups * priv_bytes_per_wg bytes.  The duration is what the load path alone needs for
 * that GEMM's bytes.  `sink` is 16 bytes of device scratch.  Asynchronous on `hip_stream`. */
int ssd_measure_mixed_read(const void* shared, size_t shared_bytes, const void* priv, size_t priv_bytes_per_wg,
                           int work_groups, int threads, int depth, void* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SSD_MEASURE_H */
