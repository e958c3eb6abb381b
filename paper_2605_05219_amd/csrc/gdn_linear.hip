// gdn_linear: the layers' projections y = x w^T + bias on the bf16 matrix cores (see include/gdn_linear.h).
//
// One workgroup of four or eight waves makes a BM (tokens) x BN (outputs) tile, a wave its part of it as tiles of
// v_mfma_f32_32x32x16_bf16.  Both operands are read along k, so a k step of BK needs a BM x BK tile of x and a
// BN x BK tile of w; they come from memory with 16-byte buffer loads straight to LDS (no registers) into a ring of
// STAGES stages, STAGES - 1 k steps ahead of the matrix cores: one barrier per k step.  Four shapes are built:
//   0: 128 x 128 x 64, 2 stages, four waves, two workgroups per compute unit   small problems (more, smaller workgroups)
//   1: 256 x 256 x 32, 4 stages, four waves, one workgroup per compute unit: a wave holds 128 x 128 outputs in 256
//      accumulator registers: half the operand bytes per flop, from memory and from LDS, three k steps of loads in flight
//   2: 256 x 256 x 64, 2 stages, eight waves of 128 tokens x 64 outputs, two per SIMD: while one wave of a SIMD is held up
//      issuing its loads to LDS the other feeds the matrix pipe, and a barrier covers 64 of k (the default for large
//      problems; 1 is kept for comparison)
//   3: 64 x 64 x 128, 4 stages, four waves of one 32 x 32 tile: problems so small that their 64 x 64 tiles fit the chip in two
//      rounds (a 512-token out-projection: 64 workgroups of shape 0 would walk k one after the other, each step waiting for
//      its loads; 256 small workgroups with three steps of 128 in flight take 11 us against 18)
// A load to LDS writes a wave's 1 KiB contiguously (lane i at 16 i), so rows are unpadded (2 BK bytes) and bank
// conflicts are avoided by choosing WHICH 16-byte piece of its row a lane fetches: piece p of row r is stored at
// position p ^ swz(r), swz(r) = (r / rows per 256 bytes) % pieces per row, which makes the 16 lanes that read the
// same piece of 16 consecutive rows hit 16 different 16-byte bank groups.  Rows past the end of x or w read as
// zeros (the buffer descriptor ends with the matrix); they only feed outputs that are never stored.  The products
// are taken transposed (w rows as the left operand), so that a lane holds four consecutive outputs of ONE token
// and stores them with one 8- or 16-byte store.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>

#include "gdn_linear.h"

namespace gdn {
namespace linear {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));


constexpr int LIN_MAX_SEG = 8;

struct LinearArgs {
    const void* x;
    const void* w;
    const float* bias;
    void* y;
    int64_t ldx, ldw, ldy;
    int64_t T;
    int32_t N, K;
    int32_t tiles_n;
    // gdn_linear_split: the outputs go to n_seg destinations by column range; n_seg = 0: everything to y
    int32_t n_seg;
    int32_t seg_col[LIN_MAX_SEG + 1];   // segment s holds outputs seg_col[s] .. seg_col[s + 1] - 1
    void* seg_y[LIN_MAX_SEG];
    int64_t seg_ld[LIN_MAX_SEG];
};

inline int32_t hip_err(hipError_t e) { return e == hipSuccess ? GDN_OK : GDN_ERR_HIP - (int32_t)e; }

// s_waitcnt vmcnt(N) (gfx9 encoding: vmcnt in bits 3:0 and 15:14; other counters left alone)
template <int N>
__device__ __forceinline__ void wait_vm() {
    __builtin_amdgcn_s_waitcnt(((N & 0x30) << 10) | (N & 0xF) | 0x0F70);
}

template <int BM_, int BN_, int BK_, int STAGES_, int WGS_PER_CU_, int WAVES_M_, int WAVES_N_>
struct LinCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, STAGES = STAGES_, WGS_PER_CU = WGS_PER_CU_;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, NW = WAVES_M * WAVES_N, THREADS = 64 * NW;   // the wave grid over the tile
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;   // a wave's tokens and outputs
    static constexpr int RB = BK * 2;                  // bytes of a tile row
    static constexpr int PP = RB / 16;                 // 16-byte pieces per row
    static constexpr int RL = 256 / RB;                // rows per 256 bytes (the span of the 64 banks)
    static constexpr int ROWS_PER_LOAD = 1024 / RB;    // rows a wave-wide load covers
    static constexpr int X_BYTES = BM * RB, W_BYTES = BN * RB, STAGE_BYTES = X_BYTES + W_BYTES;
    static constexpr int SMEM = STAGES * STAGE_BYTES;
    static constexpr int TI = WM / 32, TJ = WN / 32;   // 32 x 32 tiles of a wave along tokens / outputs
    static constexpr int XL = BM / ROWS_PER_LOAD / NW, WL = BN / ROWS_PER_LOAD / NW;   // loads per wave and stage
    static constexpr int LPS = XL + WL;
    static constexpr int AHEAD = (STAGES - 2) * LPS;   // loads that may still be in flight when a stage is handed over
    static_assert(PP * RL == 16 && (STAGES - 1) * LPS < 64 && SMEM <= 160 * 1024 && (BK / 16) % 2 == 0 &&
                  ((TI * TJ) % LPS == 0 || LPS % (TI * TJ) == 0) && XL >= 1 && WL >= 1, "tile shape");
};
typedef LinCfg<128, 128, 64, 2, 2, 2, 2> LinSmall;
typedef LinCfg<256, 256, 32, 4, 1, 2, 2> LinBig;      // four waves, 128 x 128 outputs each
typedef LinCfg<256, 256, 64, 2, 1, 2, 4> LinBig8;     // eight waves, 128 tokens x 64 outputs each: two waves per SIMD
typedef LinCfg<64, 64, 128, 4, 1, 2, 2> LinTiny;      // four waves of one 32 x 32 tile each, three k steps of 128 in flight

// The loads of one wave for one stage: 1 KiB each, XL of its quarter of the x tile, then WL of the w tile.
template <typename CFG>
struct LinLoad {
    static __device__ __forceinline__ void one(int j, char* smem, int stage, int k0, int wave, const char* xb, int x_bytes, const char* wb,
                                               int w_bytes, const int* xoff, const int* woff) {
        // buffer descriptors that end with the matrices: rows past T or N arrive as zeros
        char* xs = smem + stage * CFG::STAGE_BYTES;
        char* ws = xs + CFG::X_BYTES;
        if (j < CFG::XL) {
            const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(xb), 0, x_bytes, 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(xs + ((CFG::BM / CFG::NW) * wave + CFG::ROWS_PER_LOAD * j) * CFG::RB), 16, xoff[j], k0 * 2, 0, 0);
        } else {
            const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(wb), 0, w_bytes, 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (__attribute__((address_space(3))) void*)(ws + ((CFG::BN / CFG::NW) * wave + CFG::ROWS_PER_LOAD * (j - CFG::XL)) * CFG::RB), 16, woff[j - CFG::XL], k0 * 2, 0, 0);
        }
    }
    static __device__ __forceinline__ void all(char* smem, int stage, int k0, int wave, const char* xb, int x_bytes, const char* wb, int w_bytes,
                                               const int* xoff, const int* woff) {
#pragma unroll
        for (int j = 0; j < CFG::LPS; ++j) one(j, smem, stage, k0, wave, xb, x_bytes, wb, w_bytes, xoff, woff);
    }
};

template <typename CFG, bool OUT_BF16>
__global__ void __launch_bounds__(CFG::THREADS) __attribute__((amdgpu_waves_per_eu(CFG::WGS_PER_CU * CFG::NW / 4, CFG::WGS_PER_CU * CFG::NW / 4)))
gdn_linear_kernel(LinearArgs a) {
    constexpr int BM = CFG::BM, BN = CFG::BN, BK = CFG::BK, STAGES = CFG::STAGES, RB = CFG::RB, PP = CFG::PP, RL = CFG::RL;
    constexpr int RPL = CFG::ROWS_PER_LOAD, TI = CFG::TI, TJ = CFG::TJ, XL = CFG::XL, WL = CFG::WL;
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / CFG::WAVES_N, wn = wave % CFG::WAVES_N;   // the wave's part: tokens WM wm .., outputs WN wn ..
    const int lr = lane & 31, g = lane >> 5;
    const int tile_m = (int)blockIdx.x / a.tiles_n, tile_n = (int)blockIdx.x % a.tiles_n;
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;

    const int64_t rows_x = a.T - m0 < BM ? a.T - m0 : BM;
    const int rows_w = a.N - n0 < BN ? a.N - n0 : BN;
    const char* xb = reinterpret_cast<const char*>(a.x) + m0 * a.ldx * 2;
    const char* wb = reinterpret_cast<const char*>(a.w) + (int64_t)n0 * a.ldw * 2;
    const int x_bytes = (int)((rows_x - 1) * a.ldx * 2 + (int64_t)a.K * 2), w_bytes = (int)((int64_t)(rows_w - 1) * a.ldw * 2 + (int64_t)a.K * 2);

    // a wave-wide load writes RPL rows of RB bytes: lane i lands at row i / PP, position i % PP, and fetches the piece that belongs there
    const int ld_row = lane / PP, ld_pos = lane % PP;
    int xoff[XL], woff[WL];      // byte offsets (k = 0) of the loads this wave issues per stage
#pragma unroll
    for (int j = 0; j < XL; ++j) {
        const int row = (BM / CFG::NW) * wave + RPL * j + ld_row;
        xoff[j] = (int)(row * a.ldx * 2) + ((ld_pos ^ ((row / RL) % PP)) << 4);
    }
#pragma unroll
    for (int j = 0; j < WL; ++j) {
        const int row = (BN / CFG::NW) * wave + RPL * j + ld_row;
        woff[j] = (int)(row * a.ldw * 2) + ((ld_pos ^ ((row / RL) % PP)) << 4);
    }
    f32x16 acc[TJ][TI];          // [output tile][token tile]: lane = token, register 4 b + e = output 8 b + 4 g + e
#pragma unroll
    for (int i = 0; i < TJ; ++i)
#pragma unroll
        for (int j = 0; j < TI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // fragment reads: row r of a tile, piece 2 kk + g, stored at (2 kk + g) ^ swz(r); tile origins are multiples of 16 rows
    const int sw = (lr % 16) / RL;
    const int xrow = (CFG::WM * wm + lr) * RB, wrow = (CFG::WN * wn + lr) * RB;
    const int n_steps = a.K / BK;
    constexpr int KK = BK / 16;              // matrix-instruction steps per stage (2 or 4)
    // The stages are consumed through two fragment sets: while the matrix cores work on one k step of 16, the fragments of
    // the next are read from LDS, also across the stage boundary.  The hand-over of a stage therefore sits before the LAST
    // k step of the stage in front of it: wait for this wave's loads of the next stage, for its own fragment reads, then the
    // barrier; after it the next stage is readable by every wave and the current one (whose last fragments are in
    // registers) is free and is refilled with the stage STAGES ahead.
    bf16x8 xf[2][TI], wf[2][TJ];
    auto read_frags = [&](int stage, int kk, int set) {
        const char* xs = smem + stage * CFG::STAGE_BYTES;
        const char* ws = xs + CFG::X_BYTES;
        const int pos = ((2 * kk + g) ^ sw) * 16;
#pragma unroll
        for (int t = 0; t < TI; ++t) xf[set][t] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xs + xrow + 32 * t * RB + pos));
#pragma unroll
        for (int t = 0; t < TJ; ++t) wf[set][t] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(ws + wrow + 32 * t * RB + pos));
    };
    // Loads are issued for every stage slot, also past the last k step: there the descriptor is empty (no lane is in
    // range, nothing is fetched), so that the number of loads in flight, and with it every wait below, is the same in
    // every round and the loop body has no branch for the scheduler to stop at.
    auto mma_all = [&](int set) {
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
            for (int ti = 0; ti < TI; ++ti)
                acc[tj][ti] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[set][tj], xf[set][ti], acc[tj][ti], 0, 0, 0);
    };
#pragma unroll
    for (int p = 0; p < STAGES; ++p) {
        const bool live = p < n_steps;
        LinLoad<CFG>::all(smem, p, p * BK, wave, xb, live ? x_bytes : 0, wb, live ? w_bytes : 0, xoff, woff);
    }
    wait_vm<(STAGES - 1) * CFG::LPS>();
    __syncthreads();
    read_frags(0, 0, 0);
    int stage = 0;                           // step % STAGES
    for (int step = 0; step + 1 < n_steps; ++step) {
        const int next_stage = stage + 1 == STAGES ? 0 : stage + 1;
#pragma unroll
        for (int kk = 0; kk + 1 < KK; ++kk) {
            // The fragments of k step kk + 1 go into the other register set while the matrix instructions of k step kk are
            // issued, one read behind every matrix instruction or two, pinned in that order: left to itself the scheduler
            // reads them into the registers the matrix instructions have just used, behind them, and waits out the LDS
            // latency with the matrix pipe idle; and a burst of reads in front keeps the issue port from the matrix pipe.
            const int rs = (kk & 1) ^ 1, ms = kk & 1;
            const char* xs = smem + stage * CFG::STAGE_BYTES;
            const char* ws = xs + CFG::X_BYTES;
            const int pos = ((2 * (kk + 1) + g) ^ sw) * 16;
            constexpr int NM = TI * TJ, NR = TI + TJ;
            constexpr int SLOTS = NM < NR ? NM : NR;
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) {
#pragma unroll
                for (int q = i * NM / SLOTS; q < (i + 1) * NM / SLOTS; ++q)
                    acc[q / TI][q % TI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ms][q / TI], xf[ms][q % TI], acc[q / TI][q % TI], 0, 0, 0);
#pragma unroll
                for (int r = i * NR / SLOTS; r < (i + 1) * NR / SLOTS; ++r) {
                    if (r < TI) xf[rs][r] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xs + xrow + 32 * r * RB + pos));
                    else wf[rs][r - TI] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(ws + wrow + 32 * (r - TI) * RB + pos));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // (the matrix instructions above stay above: left to itself the scheduler sinks them below the barrier, and the
        // fragment reads and the barrier are then waited for with the matrix pipe idle)
        __builtin_amdgcn_sched_barrier(0);
        // the next stage has landed for this wave (the STAGES - 2 stages behind it may still be in flight) ...
        wait_vm<CFG::AHEAD>();
        __builtin_amdgcn_s_waitcnt(0xC07F);          // ... and this wave's last fragment reads of the current stage are done (lgkmcnt(0))
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        {
            // The last k step of the stage (fragment set 1; KK is even), written out in issue order and pinned there: a load
            // to LDS takes tens of cycles to issue, so one goes out behind every few matrix instructions, which covers it;
            // the fragments of the next stage's first k step are read in between as well.
            const bool live = step + STAGES < n_steps;
            const int xbytes = live ? x_bytes : 0, wbytes = live ? w_bytes : 0;
            const char* xs = smem + next_stage * CFG::STAGE_BYTES;
            const char* ws = xs + CFG::X_BYTES;
            const int pos = (g ^ sw) * 16;
            constexpr int NM = TI * TJ, NL = CFG::LPS, NR = TI + TJ;
            constexpr int SLOTS = NM < NL ? NM : NL;             // interleave slots
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) {
#pragma unroll
                for (int q = i * NM / SLOTS; q < (i + 1) * NM / SLOTS; ++q)
                    acc[q / TI][q % TI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1][q / TI], xf[1][q % TI], acc[q / TI][q % TI], 0, 0, 0);
#pragma unroll
                for (int r = i * NR / SLOTS; r < (i + 1) * NR / SLOTS; ++r) {
                    if (r < TI) xf[0][r] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xs + xrow + 32 * r * RB + pos));
                    else wf[0][r - TI] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(ws + wrow + 32 * (r - TI) * RB + pos));
                }
#pragma unroll
                for (int j = i * NL / SLOTS; j < (i + 1) * NL / SLOTS; ++j)
                    LinLoad<CFG>::one(j, smem, stage, (step + STAGES) * BK, wave, xb, xbytes, wb, wbytes, xoff, woff);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        stage = next_stage;
    }
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {        // the last stage: nothing behind it
        if (kk + 1 < KK) read_frags(stage, kk + 1, (kk & 1) ^ 1);
        mma_all(kk & 1);
    }

    // ---- epilogue: bias, one rounding, and out through LDS.  A lane holds runs of four outputs of ONE token, 32 tokens per
    //      instruction: stored from there, every instruction would touch 32 rows of the output with 8 or 16 bytes each.
    //      Each wave turns its quarter around in its own quarter of the (now idle) stage ring instead: rows of 256 bytes (128
    //      with the small tile), the 16-byte pieces of a row XOR-swizzled with the token so that both the writes (lane = token)
    //      and the reads (lane = piece) spread over the banks; then 16 lanes store one row's 256 contiguous bytes.  A wave's LDS
    //      operations execute in order, so no barrier stands between its writes and reads; the one barrier before keeps the
    //      other waves' last fragment reads out of the way.
    constexpr int ES = OUT_BF16 ? 2 : 4;
    constexpr int WN = CFG::WN, WM = CFG::WM;                      // the wave's outputs and tokens
    constexpr int REGION = CFG::SMEM / CFG::NW;                    // the wave's part of the ring
    constexpr int PW = (WN * ES <= 256) ? WN : 256 / ES;           // outputs per pass: a row of at most 256 bytes
    constexpr int RBY = PW * ES, PPR = RBY / 16;                   // row bytes, 16-byte pieces per row
    constexpr int RPI = 1024 / RBY;                                // rows a wave-wide 16-byte access covers
    constexpr int TP = (WM * RBY <= REGION) ? WM : REGION / RBY;   // tokens per pass
    static_assert(TP % 32 == 0 && TP >= 32 && WM % TP == 0 && WN % PW == 0 && PW % 32 == 0, "epilogue region");
    wait_vm<0>();
    __syncthreads();
    char* const reg = smem + wave * REGION;
    const int64_t tok0 = m0 + WM * wm;
    const int col0 = n0 + WN * wn;
#pragma unroll
    for (int c0 = 0; c0 < WN; c0 += PW) {
#pragma unroll
        for (int t0 = 0; t0 < WM; t0 += TP) {
#pragma unroll
            for (int tj = c0 / 32; tj < (c0 + PW) / 32; ++tj)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int cl = 32 * tj + 8 * b + 4 * g;        // first of the lane's four outputs, within the wave's part
                    f32x4 bv = {0.f, 0.f, 0.f, 0.f};
                    if (a.bias) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col0 + cl + e < a.N) bv[e] = a.bias[col0 + cl + e];
                    }
#pragma unroll
                    for (int ti = t0 / 32; ti < (t0 + TP) / 32; ++ti) {
                        const int row = 32 * ti + lr - t0;
                        f32x4 v = {acc[tj][ti][4 * b] + bv[0], acc[tj][ti][4 * b + 1] + bv[1], acc[tj][ti][4 * b + 2] + bv[2], acc[tj][ti][4 * b + 3] + bv[3]};
                        const int byte = (cl - c0) * ES;
                        char* const dst = reg + row * RBY + (((byte >> 4) ^ (row % PPR)) << 4) + (byte & 15);
                        if (OUT_BF16) *reinterpret_cast<bf16x4*>(dst) = __builtin_convertvector(v, bf16x4);
                        else *reinterpret_cast<f32x4*>(dst) = v;
                    }
                }
#pragma unroll
            for (int i = 0; i < TP / RPI; ++i) {
                const int row = RPI * i + lane / PPR, piece = lane % PPR;
                const u32x4 val = *reinterpret_cast<const u32x4*>(reg + row * RBY + ((piece ^ (row % PPR)) << 4));
                const int64_t tok = tok0 + t0 + row;
                const int col = col0 + c0 + piece * (16 / ES);
                if (tok < a.T && col < a.N) {
                    // the destination of this piece: the whole output, or the segment its first column lies in (segment
                    // boundaries are multiples of 8 columns, so a piece lies in one segment)
                    char* base = reinterpret_cast<char*>(a.y);
                    int64_t ld = a.ldy;
                    int c_lo = 0, c_hi = a.N;
                    if (a.n_seg > 0) {
#pragma unroll
                        for (int sg = 0; sg < LIN_MAX_SEG; ++sg)
                            if (sg < a.n_seg && col >= a.seg_col[sg]) {
                                base = reinterpret_cast<char*>(a.seg_y[sg]);
                                ld = a.seg_ld[sg];
                                c_lo = a.seg_col[sg];
                                c_hi = a.seg_col[sg + 1];
                            }
                    }
                    char* const p = base + (tok * ld + (col - c_lo)) * ES;
                    if (col + 16 / ES <= c_hi) {
                        *reinterpret_cast<u32x4*>(p) = val;
                    } else {
#pragma unroll
                        for (int e = 0; e < 16 / ES; ++e)
                            if (col + e < c_hi) {
                                if (OUT_BF16) reinterpret_cast<uint16_t*>(p)[e] = (uint16_t)(val[e >> 1] >> (16 * (e & 1)));
                                else reinterpret_cast<uint32_t*>(p)[e] = val[e];
                            }
                    }
                }
            }
        }
    }
}

template <typename CFG, bool OUT_BF16>
hipError_t launch_linear(LinearArgs a, hipStream_t stream) {
    static hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_linear_kernel<CFG, OUT_BF16>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, CFG::SMEM);
    if (attr_err != hipSuccess) return attr_err;
    const int64_t tiles_m = (a.T + CFG::BM - 1) / CFG::BM;
    a.tiles_n = (a.N + CFG::BN - 1) / CFG::BN;
    hipLaunchKernelGGL((gdn_linear_kernel<CFG, OUT_BF16>), dim3((unsigned)(tiles_m * a.tiles_n)), dim3(CFG::THREADS), CFG::SMEM, stream, a);
    return hipGetLastError();
}

std::atomic<int32_t> g_linear_shape{-1};

int chip_cus_linear() {
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
            (void)hipGetLastError();
            return 256;
        }
        return cus;
    }();
    return n;
}

// Which tile shape a problem gets: the estimated time of each shape is its number of rounds of workgroups over the
// chip times the work of one workgroup over the shape's measured rate (relative figures).
int choose_linear_shape(int64_t T, int32_t N, int32_t K) {
    const int forced = g_linear_shape.load();
    if (forced >= 0) return (forced == 3 && K % 128 != 0) ? 0 : forced;      // shape 3 walks k in steps of 128
    const double cus = (double)chip_cus_linear();
    // at most two rounds of 64 x 64 tiles, one per compute unit (measured, shape 3 against shape 0: 512 x 2048 11 against 17 us,
    // 512 x 2560 19 against 23, 1024 x 2048 19 against 23; 256 x 8224, three rounds, 32 against 23)
    if (K % 128 == 0 && (double)((T + 63) / 64) * (double)((N + 63) / 64) <= 2.0 * cus) return 3;
    const struct { int id, bm, bn, per_cu; double rate; } shapes[2] = {{0, 128, 128, 2, 0.34}, {2, 256, 256, 1, 0.53}};
    int best = 0;
    double best_t = 0;
    for (int i = 0; i < 2; ++i) {
        const double wgs = (double)((T + shapes[i].bm - 1) / shapes[i].bm) * (double)((N + shapes[i].bn - 1) / shapes[i].bn);
        const double rounds = std::ceil(wgs / (cus * shapes[i].per_cu));
        const double t = rounds * shapes[i].per_cu * shapes[i].bm * shapes[i].bn / shapes[i].rate;
        if (i == 0 || t < best_t) { best = shapes[i].id; best_t = t; }
    }
    return best;
}

}  // namespace linear
}  // namespace gdn

using namespace gdn;
using namespace gdn::linear;

namespace {
int32_t linear_checks(const void* x, int64_t ldx, const void* w, int64_t ldw, const float* bias, int32_t out_dtype, int64_t T, int32_t N,
                      int32_t K) {
    if (T < 0 || N < 0 || K < 0) return GDN_ERR_COUNT;
    if (out_dtype != GDN_BF16 && out_dtype != GDN_F32) return GDN_ERR_SHAPE;
    if (K % 64 != 0 || ldx < K || ldw < K) return GDN_ERR_SHAPE;
    if (T == 0 || N == 0) return GDN_OK;
    if (K == 0) return GDN_ERR_SHAPE;
    if (!x || !w) return GDN_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(x) & 15u) || (reinterpret_cast<uintptr_t>(w) & 15u) || (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)))
        return GDN_ERR_ALIGN;
    if ((ldx & 7) || (ldw & 7)) return GDN_ERR_ALIGN;
    // a tile's rows must be addressable with 31-bit byte offsets
    if ((int64_t)256 * ldx * 2 >= ((int64_t)1 << 31) || (int64_t)256 * ldw * 2 >= ((int64_t)1 << 31)) return GDN_ERR_COUNT;
    if (((T + 127) / 128) * (((int64_t)N + 127) / 128) > INT32_MAX) return GDN_ERR_COUNT;
    return GDN_OK;
}

int32_t linear_launch(LinearArgs& a, int32_t out_dtype, hipStream_t stream) {
    a.tiles_n = 0;
    const bool bf = out_dtype == GDN_BF16;
    hipError_t e;
    switch (choose_linear_shape(a.T, a.N, a.K)) {
        case 1: e = bf ? launch_linear<LinBig, true>(a, stream) : launch_linear<LinBig, false>(a, stream); break;
        case 2: e = bf ? launch_linear<LinBig8, true>(a, stream) : launch_linear<LinBig8, false>(a, stream); break;
        case 3: e = bf ? launch_linear<LinTiny, true>(a, stream) : launch_linear<LinTiny, false>(a, stream); break;
        default: e = bf ? launch_linear<LinSmall, true>(a, stream) : launch_linear<LinSmall, false>(a, stream); break;
    }
    return hip_err(e);
}
}  // namespace

extern "C" int32_t gdn_linear(const void* x, int64_t ldx, const void* w, int64_t ldw, const float* bias, void* y, int64_t ldy,
                              int32_t out_dtype, int64_t T, int32_t N, int32_t K, void* stream_) {
    const int32_t rc = linear_checks(x, ldx, w, ldw, bias, out_dtype, T, N, K);
    if (rc != GDN_OK) return rc;
    if (ldy < N) return GDN_ERR_SHAPE;
    if (T == 0 || N == 0) return GDN_OK;
    if (!y) return GDN_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(y) & (out_dtype == GDN_BF16 ? 7u : 15u)) || (ldy & 3)) return GDN_ERR_ALIGN;
    LinearArgs a = {};
    a.x = x; a.w = w; a.bias = bias; a.y = y;
    a.ldx = ldx; a.ldw = ldw; a.ldy = ldy;
    a.T = T; a.N = N; a.K = K;
    a.n_seg = 0;
    return linear_launch(a, out_dtype, (hipStream_t)stream_);
}

extern "C" int32_t gdn_linear_split(const void* x, int64_t ldx, const void* w, int64_t ldw, const float* bias, int32_t n_seg,
                                    const int32_t* seg_cols, void* const* seg_y, const int64_t* seg_ld, int32_t out_dtype, int64_t T,
                                    int32_t K, void* stream_) {
    if (n_seg < 1 || n_seg > LIN_MAX_SEG) return GDN_ERR_COUNT;
    if (!seg_cols || !seg_y || !seg_ld) return GDN_ERR_NULL;
    if (seg_cols[0] != 0) return GDN_ERR_SHAPE;
    for (int32_t sg = 0; sg < n_seg; ++sg) {
        if (seg_cols[sg + 1] <= seg_cols[sg]) return GDN_ERR_SHAPE;                 // empty or decreasing
        if (sg + 1 < n_seg && (seg_cols[sg + 1] & 7)) return GDN_ERR_ALIGN;         // inner boundaries: whole 16-byte pieces
    }
    const int32_t N = seg_cols[n_seg];
    const int32_t rc = linear_checks(x, ldx, w, ldw, bias, out_dtype, T, N, K);
    if (rc != GDN_OK) return rc;
    for (int32_t sg = 0; sg < n_seg; ++sg) {
        if (seg_ld[sg] < seg_cols[sg + 1] - seg_cols[sg]) return GDN_ERR_SHAPE;
        if (T > 0 && !seg_y[sg]) return GDN_ERR_NULL;
        if ((reinterpret_cast<uintptr_t>(seg_y[sg]) & (out_dtype == GDN_BF16 ? 7u : 15u)) || (seg_ld[sg] & 3)) return GDN_ERR_ALIGN;
    }
    if (T == 0) return GDN_OK;
    LinearArgs a = {};
    a.x = x; a.w = w; a.bias = bias; a.y = seg_y[0];
    a.ldx = ldx; a.ldw = ldw; a.ldy = seg_ld[0];
    a.T = T; a.N = N; a.K = K;
    a.n_seg = n_seg;
    for (int32_t sg = 0; sg < n_seg; ++sg) {
        a.seg_col[sg] = seg_cols[sg];
        a.seg_y[sg] = seg_y[sg];
        a.seg_ld[sg] = seg_ld[sg];
    }
    for (int32_t sg = n_seg; sg <= LIN_MAX_SEG; ++sg) a.seg_col[sg] = N;
    return linear_launch(a, out_dtype, (hipStream_t)stream_);
}

extern "C" int32_t gdn_linear_tune(int32_t shape) {
    return g_linear_shape.exchange(shape < 0 || shape > 3 ? -1 : shape);
}
