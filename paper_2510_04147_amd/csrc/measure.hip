// Measurement kernels, built into a library of their own (libssd_measure.so): they are no part of
// the decoding path and the product library does not export them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ssd_measure.h"

// ------------------------------------------------------------------------
// Measurement aid: a pure read of `bytes` with the access pattern of the
// GEMM's weight stream (each wave walks its own contiguous region with
// 16-byte loads, DEPTH independent loads in flight).  It gives the HBM read
// rate the chip sustains for that pattern: the practical ceiling the GEMM is
// measured against.
// ------------------------------------------------------------------------
template <int DEPTH>
__global__ __launch_bounds__(512) void k_stream_read(const uint4* src, size_t n16_per_wave, unsigned* sink) {
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const uint4* p = src + wave * n16_per_wave + lane;
    unsigned acc = 0;
    for (size_t i = 0; i < n16_per_wave; i += 64 * DEPTH) {
        uint4 v[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) v[d] = p[i + (size_t)d * 64];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) acc ^= v[d].x ^ v[d].y ^ v[d].z ^ v[d].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;      // practically never true; keeps the loads alive
}

extern "C" __attribute__((visibility("default"))) int ssd_measure_stream_read(const void* src, size_t bytes,
                                                                            int work_groups, int waves_per_wg,
                                                                            int depth, void* sink, void* stream) {
    if (!src || !sink || work_groups < 1 || waves_per_wg < 1 || waves_per_wg > 8) return -1;
    const size_t waves = (size_t)work_groups * waves_per_wg;
    size_t per = bytes / 16 / waves;
    per -= per % (64 * 16);                      // whole unrolled steps for every depth
    if (per == 0) return -1;
    hipStream_t st = (hipStream_t)stream;
    if (depth == 16)
        k_stream_read<16><<<work_groups, waves_per_wg * 64, 0, st>>>((const uint4*)src, per, (unsigned*)sink);
    else if (depth == 8)
        k_stream_read<8><<<work_groups, waves_per_wg * 64, 0, st>>>((const uint4*)src, per, (unsigned*)sink);
    else if (depth == 4)
        k_stream_read<4><<<work_groups, waves_per_wg * 64, 0, st>>>((const uint4*)src, per, (unsigned*)sink);
    else
        return -1;
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

// ------------------------------------------------------------------------
// Measurement aid: the loads of a weight-streaming GEMM and nothing else.  Every work-group reads
// the SAME `shared` buffer once (the activations, served by L2) and its OWN slice of `priv` (its share
// of the weights, from HBM, non-temporal like the GEMM's), interleaved evenly, 4 x 16 bytes in
// flight per lane (DEPTH 4; or 8, and 512 or 1024 lanes).  Its duration is what the load path alone needs
// for a GEMM's bytes in a one-tile-per-CU decomposition: the floor of such a kernel whatever its arithmetic costs.
// ------------------------------------------------------------------------
typedef unsigned int mr_u32x4 __attribute__((ext_vector_type(4)));
template <int DEPTH, int THREADS>
__global__ __launch_bounds__(THREADS) void k_mixed_read(const mr_u32x4* __restrict__ shared, int steps_s,
                                                        const mr_u32x4* __restrict__ priv, int steps_p, unsigned* sink) {
    const int tid = threadIdx.x;
    const mr_u32x4* pp = priv + (size_t)blockIdx.x * steps_p * DEPTH * THREADS;
    unsigned acc = 0;
    int ip = 0;
    for (int is = 0; is < steps_s; ++is) {
        mr_u32x4 v[DEPTH], w[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) v[d] = shared[((size_t)is * DEPTH + d) * THREADS + tid];
        // private steps spread evenly over the shared ones: those whose index falls into this interval
        const int hi = (int)(((long long)(is + 1) * steps_p) / steps_s);
        for (; ip < hi; ++ip) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) w[d] = __builtin_nontemporal_load(&pp[((size_t)ip * DEPTH + d) * THREADS + tid]);
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) acc ^= w[d].x ^ w[d].y ^ w[d].z ^ w[d].w;
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) acc ^= v[d].x ^ v[d].y ^ v[d].z ^ v[d].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;      // practically never true; keeps the loads alive
}

extern "C" __attribute__((visibility("default"))) int ssd_measure_mixed_read(const void* shared, size_t shared_bytes,
                                                                           const void* priv, size_t priv_bytes_per_wg,
                                                                           int work_groups, int threads, int depth,
                                                                           void* sink, void* stream) {
    if ((threads != 512 && threads != 1024) || (depth != 4 && depth != 8)) return -1;
    const size_t step = (size_t)threads * depth * 16;            // bytes one work-group reads per step
    if (!shared || !priv || !sink || work_groups < 1 || shared_bytes < step || shared_bytes % step ||
        priv_bytes_per_wg % step || shared_bytes / step > (1u << 20) || priv_bytes_per_wg / step > (1u << 20))
        return -1;
    const int ss = (int)(shared_bytes / step), sp = (int)(priv_bytes_per_wg / step);
    hipStream_t st = (hipStream_t)stream;
    const mr_u32x4 *a = (const mr_u32x4*)shared, *b = (const mr_u32x4*)priv;
    if (threads == 512 && depth == 4) k_mixed_read<4, 512><<<work_groups, 512, 0, st>>>(a, ss, b, sp, (unsigned*)sink);
    else if (threads == 512) k_mixed_read<8, 512><<<work_groups, 512, 0, st>>>(a, ss, b, sp, (unsigned*)sink);
    else if (depth == 4) k_mixed_read<4, 1024><<<work_groups, 1024, 0, st>>>(a, ss, b, sp, (unsigned*)sink);
    else k_mixed_read<8, 1024><<<work_groups, 1024, 0, st>>>(a, ss, b, sp, (unsigned*)sink);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
