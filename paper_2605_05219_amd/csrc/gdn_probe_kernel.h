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

// dst[i] = src[i]: one non-temporal 16-byte access each way per thread, a workgroup per 4 KiB (the form that moves the most
// bytes per second on this chip: see ckpt_copy_kernel).
__global__ void __launch_bounds__(PROBE_THREADS) probe_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst,
                                                                   int64_t n4) {
    const int64_t i = (int64_t)blockIdx.x * PROBE_THREADS + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace gdn
