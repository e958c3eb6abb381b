// gdn_linear: the layers' projections y = x w^T + bias on the bf16 matrix cores (see include/gdn_linear.h).
//
// One workgroup of four waves makes a 128 (tokens) x 128 (outputs) tile; a wave a 64 x 64 quarter as 2 x 2
// accumulator tiles of v_mfma_f32_32x32x16_bf16.  Both operands are read along k, so a tile of x and a tile of w
// (128 rows x 64 k each, 16 KiB) are what a k step of 64 needs; they come from memory with 16-byte buffer loads
// straight to LDS (no registers), into the other of two stages while the matrix cores work on this one: one
// barrier per k step.  A load to LDS writes a wave's 1 KiB contiguously (lane i at 16 i), so rows are unpadded
// (128 bytes) and bank conflicts are avoided by choosing WHICH 16-byte piece of its row a lane fetches: piece p of
// row r is stored at position p ^ ((r >> 1) & 7), which makes the 16 lanes of a fragment read (16 consecutive rows,
// the same piece) hit 16 different 16-byte bank groups.  Rows past the end of x or w read as zeros (the buffer
// descriptor ends with the matrix).  The products are taken transposed (w rows as the left operand), so that a
// lane holds four consecutive outputs of ONE token and stores them with one 8- or 16-byte store.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "gdn_linear.h"

namespace gdn {
namespace {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int LIN_BM = 128, LIN_BN = 128, LIN_BK = 64, LIN_THREADS = 256;
constexpr int LIN_TILE_BYTES = LIN_BM * LIN_BK * 2;        // 16 KiB: one operand tile of one stage
constexpr int LIN_SMEM = 4 * LIN_TILE_BYTES;               // x and w tiles, two stages

struct LinearArgs {
    const void* x;
    const void* w;
    const float* bias;
    void* y;
    int64_t ldx, ldw, ldy;
    int64_t T;
    int32_t N, K;
    int32_t tiles_n;
};

inline int32_t hip_err(hipError_t e) { return e == hipSuccess ? GDN_OK : GDN_ERR_HIP - (int32_t)e; }

__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

template <bool OUT_BF16>
__global__ void __launch_bounds__(LIN_THREADS) gdn_linear_kernel(LinearArgs a) {
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;                 // the wave's quarter: tokens 64 wm .., outputs 64 wn ..
    const int lr = lane & 31, g = lane >> 5;
    const int tile_m = (int)blockIdx.x / a.tiles_n, tile_n = (int)blockIdx.x % a.tiles_n;
    const int64_t m0 = (int64_t)tile_m * LIN_BM;
    const int n0 = tile_n * LIN_BN;

    // buffer descriptors that end with the matrices: rows past T or N arrive as zeros
    const int64_t rows_x = a.T - m0 < LIN_BM ? a.T - m0 : LIN_BM;
    const int rows_w = a.N - n0 < LIN_BN ? a.N - n0 : LIN_BN;
    const char* xb = reinterpret_cast<const char*>(a.x) + m0 * a.ldx * 2;
    const char* wb = reinterpret_cast<const char*>(a.w) + (int64_t)n0 * a.ldw * 2;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(xb), 0, (int)((rows_x - 1) * a.ldx * 2 + a.K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(wb), 0, (int)((int64_t)(rows_w - 1) * a.ldw * 2 + a.K * 2), 0x00020000);

    // a wave-wide load writes 8 rows of 128 bytes: lane i lands at row i / 8, position i % 8, and fetches the piece that belongs there
    const int ld_row = lane >> 3, ld_pos = lane & 7;
    int xoff[4], woff[4];        // byte offsets (k = 0) of the 4 loads per operand this wave issues per stage: rows 32 wave + 8 j ..
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 32 * wave + 8 * j + ld_row;
        const int piece = ld_pos ^ ((row >> 1) & 7);
        xoff[j] = (int)(row * a.ldx * 2) + piece * 16;
        woff[j] = (int)(row * a.ldw * 2) + piece * 16;
    }
    auto issue = [&](int stage, int k0) {
        char* xs = smem + stage * 2 * LIN_TILE_BYTES;
        char* ws = xs + LIN_TILE_BYTES;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(xs + (32 * wave + 8 * j) * 128), 16, xoff[j], k0 * 2, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (__attribute__((address_space(3))) void*)(ws + (32 * wave + 8 * j) * 128), 16, woff[j], k0 * 2, 0, 0);
        }
    };

    f32x16 acc[2][2];            // [output tile tj][token tile ti]: lane = token, register 4 b + e = output 8 b + 4 g + e
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // fragment read offsets: row r of a tile, piece 2 kk + g, stored at (2 kk + g) ^ ((r >> 1) & 7)
    const int sw = (lr >> 1) & 7;            // the same for rows r + 32 ti (32 >> 1 = 16 keeps the low three bits)
    const int n_steps = a.K / LIN_BK;
    issue(0, 0);
    for (int step = 0; step < n_steps; ++step) {
        const int stage = step & 1;
        wait_vm0();                          // this stage has landed (nothing else is in flight)
        __syncthreads();                     // ... for every wave, and every wave is done with the other stage
        if (step + 1 < n_steps) issue(stage ^ 1, (step + 1) * LIN_BK);
        const char* xs = smem + stage * 2 * LIN_TILE_BYTES;
        const char* ws = xs + LIN_TILE_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int pos = ((2 * kk + g) ^ sw) * 16;
            bf16x8 xf[2], wf[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                xf[t] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xs + (64 * wm + 32 * t + lr) * 128 + pos));
                wf[t] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(ws + (64 * wn + 32 * t + lr) * 128 + pos));
            }
#pragma unroll
            for (int tj = 0; tj < 2; ++tj)
#pragma unroll
                for (int ti = 0; ti < 2; ++ti)
                    acc[tj][ti] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[tj], xf[ti], acc[tj][ti], 0, 0, 0);
        }
    }

    // ---- epilogue: bias, one rounding, 4 consecutive outputs of a token per store
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
        const int64_t tok = m0 + 64 * wm + 32 * ti + lr;
        if (tok >= a.T) continue;
#pragma unroll
        for (int tj = 0; tj < 2; ++tj)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int col = n0 + 64 * wn + 32 * tj + 8 * b + 4 * g;
                if (col >= a.N) continue;
                f32x4 v = {acc[tj][ti][4 * b], acc[tj][ti][4 * b + 1], acc[tj][ti][4 * b + 2], acc[tj][ti][4 * b + 3]};
                const bool whole = col + 4 <= a.N;
                if (a.bias) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < a.N) v[e] += a.bias[col + e];
                }
                if (OUT_BF16) {
                    __bf16* p = reinterpret_cast<__bf16*>(a.y) + tok * a.ldy + col;
                    const bf16x4 h = __builtin_convertvector(v, bf16x4);
                    if (whole) *reinterpret_cast<bf16x4*>(p) = h;
                    else
                        for (int e = 0; e < 4; ++e)
                            if (col + e < a.N) p[e] = h[e];
                } else {
                    float* p = reinterpret_cast<float*>(a.y) + tok * a.ldy + col;
                    if (whole) *reinterpret_cast<f32x4*>(p) = v;
                    else
                        for (int e = 0; e < 4; ++e)
                            if (col + e < a.N) p[e] = v[e];
                }
            }
    }
}

}  // namespace
}  // namespace gdn

using namespace gdn;

extern "C" int32_t gdn_linear(const void* x, int64_t ldx, const void* w, int64_t ldw, const float* bias, void* y, int64_t ldy,
                              int32_t out_dtype, int64_t T, int32_t N, int32_t K, void* stream_) {
    if (T < 0 || N < 0 || K < 0) return GDN_ERR_COUNT;
    if (out_dtype != GDN_BF16 && out_dtype != GDN_F32) return GDN_ERR_SHAPE;
    if (K % LIN_BK != 0 || ldx < K || ldw < K || ldy < N) return GDN_ERR_SHAPE;
    if (T == 0 || N == 0) return GDN_OK;
    if (K == 0) return GDN_ERR_SHAPE;
    if (!x || !w || !y) return GDN_ERR_NULL;
    const uintptr_t ya = out_dtype == GDN_BF16 ? 7u : 15u;
    if ((reinterpret_cast<uintptr_t>(x) & 15u) || (reinterpret_cast<uintptr_t>(w) & 15u) || (reinterpret_cast<uintptr_t>(y) & ya) ||
        (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)))
        return GDN_ERR_ALIGN;
    if ((ldx & 7) || (ldw & 7) || (ldy & 3)) return GDN_ERR_ALIGN;
    // a tile's rows must be addressable with 31-bit byte offsets
    if ((int64_t)LIN_BM * ldx * 2 >= ((int64_t)1 << 31) || (int64_t)LIN_BN * ldw * 2 >= ((int64_t)1 << 31)) return GDN_ERR_COUNT;
    const int64_t tiles_m = (T + LIN_BM - 1) / LIN_BM;
    const int64_t tiles_n = (N + LIN_BN - 1) / LIN_BN;
    if (tiles_m * tiles_n > INT32_MAX) return GDN_ERR_COUNT;
    LinearArgs a;
    a.x = x; a.w = w; a.bias = bias; a.y = y;
    a.ldx = ldx; a.ldw = ldw; a.ldy = ldy;
    a.T = T; a.N = N; a.K = K;
    a.tiles_n = (int32_t)tiles_n;
    hipStream_t stream = (hipStream_t)stream_;
    const dim3 grid((unsigned)(tiles_m * tiles_n));
    static hipError_t attr_err = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_linear_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize, LIN_SMEM);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_linear_kernel<false>), hipFuncAttributeMaxDynamicSharedMemorySize, LIN_SMEM);
        return e;
    }();
    if (attr_err != hipSuccess) return hip_err(attr_err);
    if (out_dtype == GDN_BF16) hipLaunchKernelGGL(gdn_linear_kernel<true>, grid, dim3(LIN_THREADS), LIN_SMEM, stream, a);
    else hipLaunchKernelGGL(gdn_linear_kernel<false>, grid, dim3(LIN_THREADS), LIN_SMEM, stream, a);
    return hip_err(hipGetLastError());
}
