// Machine ceilings measured on the spot (not a step of the method): an MFMA loop and a plain
// copy, so that a roofline fraction can be read against what this chip delivers and not only
// against the data-sheet peaks.
#pragma once
#include <hip/hip_runtime.h>

#include "gdn_mma.h"

namespace gdn {

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_MFMA_PER_ITER = 8;   // eight independent accumulators per wave

// Every wave issues iters x 8 v_mfma_f32_32x32x16_f16 on independent accumulators with operands
// that never change; the sums land in out[block * 256 + thread] so the loop is kept.
__global__ void __launch_bounds__(PROBE_THREADS) probe_mfma_kernel(float* __restrict__ out, int iters) {
    typedef Elem<half_t> EL;
    typename EL::Frag fa, fb;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        fa[e] = (half_t)(0.001f * (float)((lane + e) & 7));
        fb[e] = (half_t)(0.002f * (float)((lane ^ e) & 3));
    }
    f32x16 acc[PROBE_MFMA_PER_ITER];
#pragma unroll
    for (int j = 0; j < PROBE_MFMA_PER_ITER; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < PROBE_MFMA_PER_ITER; ++j) acc[j] = EL::mma(fa, fb, acc[j]);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < PROBE_MFMA_PER_ITER; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    out[(int64_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

// dst[i] = src[i], 16 bytes per access; a workgroup moves contiguous 16 KiB tiles, four loads in
// flight per thread.
__global__ void __launch_bounds__(PROBE_THREADS) probe_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                                   int64_t n4) {
    constexpr int64_t TILE = 4 * PROBE_THREADS;
    const int64_t n_tiles = n4 / TILE;
    for (int64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const int64_t base = t * TILE + threadIdx.x;
        float4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = src[base + u * PROBE_THREADS];
#pragma unroll
        for (int u = 0; u < 4; ++u) dst[base + u * PROBE_THREADS] = x[u];
    }
    if (blockIdx.x == 0)
        for (int64_t i = n_tiles * TILE + threadIdx.x; i < n4; i += PROBE_THREADS) dst[i] = src[i];
}

}  // namespace gdn
