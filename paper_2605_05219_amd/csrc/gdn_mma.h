// Matrix-core building blocks for gfx950 (wave64), shared by the prep and recurrence kernels.
//
// Every contraction here is D[m][n] += sum_k X[m][k] * Y[n][k] on a 32x32 output tile per wave,
// with both operands read row-wise along k.  Lane l supplies row (l & 31) of X as the MFMA's A
// operand and row (l & 31) of Y as its B operand; its half-wave index g = l >> 5 selects which
// k-slots of the step it carries.  The hardware only pairs slot with slot, so the order in
// which contraction indices are assigned to slots is free as long as A and B agree.  The
// order used everywhere is the one the accumulator layout induces: accumulator register
// 4b+e of lane (n, g) holds output row 8b+4g+e of column n.  With it, an accumulator tile
// whose ROWS are the next contraction's index can be fed back as a B operand straight from
// registers, with no shuffle and no trip through LDS:
//   fp16: step s of a 32-row tile uses registers 8s..8s+7, i.e. rows 16s+4g+{0..3} and
//         16s+8+4g+{0..3}; an operand read from memory loads exactly those two 4-element runs.
//   fp32: step 4b+e uses register 4b+e, i.e. row 8b+4g+e.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gdn {

typedef _Float16 half_t;
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Makes a value opaque to the optimiser at this point (an empty statement that "modifies" it).
// Two uses: pure arithmetic stays where it is written, next to the matrix instruction it is
// meant to hide under (the statement is ordered with the scheduling fences); and addresses
// derived from an opaque coordinate cannot be hoisted out of a loop into registers of their own.
template <typename T>
__device__ __forceinline__ void pin(T& x) { asm volatile("" : "+v"(x)); }

// Output row (within a 32x32 tile) held by accumulator register idx of half-wave g.
// Inclusive running sum over the 64 lanes of a wave by cross-lane adds only (no LDS traffic):
// shifts by 1, 2, 4 and 8 inside each row of 16 lanes with zeros shifted in, then lane 15 of
// rows 0 and 2 added to the row above, then lane 31 added to the upper half.  All lanes active.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or_zero(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xF, true));
}
__device__ __forceinline__ float wave_running_sum(float x) {
    x += dpp_or_zero<0x111, 0xF>(x);   // row_shr:1
    x += dpp_or_zero<0x112, 0xF>(x);   // row_shr:2
    x += dpp_or_zero<0x114, 0xF>(x);   // row_shr:4
    x += dpp_or_zero<0x118, 0xF>(x);   // row_shr:8
    x += dpp_or_zero<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
    x += dpp_or_zero<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3
    return x;
}
__device__ __forceinline__ float wave_last_lane(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

__device__ __forceinline__ int acc_row(int idx, int g) { return 8 * (idx >> 2) + 4 * g + (idx & 3); }

template <typename E> struct Elem;

template <> struct Elem<half_t> {
    typedef uint16_t In;               // bf16 bits in global memory
    typedef half8 Frag;
    static constexpr int PAD = 4;      // row padding (elements) of LDS tiles: 2 dwords, keeps 8-byte alignment
    static constexpr int KSTEP = 16;   // contraction indices per MFMA
    static constexpr int STEPS_PER_TILE = 2;  // MFMA steps that consume one 32-row accumulator tile

    // slot4: where the 4-aligned run of contraction indices starting at c is stored in an LDS row
    // (the identity: rows are kept in index order and a step's operand is two 8-byte reads)
    static __device__ __forceinline__ int slot4(int c) { return c; }
    static __device__ __forceinline__ Frag load(const half_t* row, int s, int g) {
        const half4 lo = *reinterpret_cast<const half4*>(row + 16 * s + 4 * g);
        const half4 hi = *reinterpret_cast<const half4*>(row + 16 * s + 8 + 4 * g);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    // f[slot] * vec[index that slot carries]  (vec indexed like a row handed to load())
    static __device__ __forceinline__ Frag scale(Frag f, const float* vec, int s, int g) {
        const f32x4 lo = *reinterpret_cast<const f32x4*>(vec + 16 * s + 4 * g);
        const f32x4 hi = *reinterpret_cast<const f32x4*>(vec + 16 * s + 8 + 4 * g);
        Frag r;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            r[e] = (half_t)((float)f[e] * lo[e]);
            r[4 + e] = (half_t)((float)f[4 + e] * hi[e]);
        }
        return r;
    }
    static __device__ __forceinline__ Frag from_acc(const f32x16& acc, int sub) {
        Frag f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (half_t)acc[8 * sub + e];
        return f;
    }
    // the operand fragment load() would return for the row (x[c] * vec[c])_c, x and vec fp32 in LDS
    static __device__ __forceinline__ Frag load_scaled(const float* x, const float* vec, int s, int g) {
        const f32x4 lo = *reinterpret_cast<const f32x4*>(x + 16 * s + 4 * g);
        const f32x4 hi = *reinterpret_cast<const f32x4*>(x + 16 * s + 8 + 4 * g);
        const f32x4 vl = *reinterpret_cast<const f32x4*>(vec + 16 * s + 4 * g);
        const f32x4 vh = *reinterpret_cast<const f32x4*>(vec + 16 * s + 8 + 4 * g);
        Frag f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[e] = (half_t)(lo[e] * vl[e]);
            f[4 + e] = (half_t)(hi[e] * vh[e]);
        }
        return f;
    }
    static __device__ __forceinline__ void store4(half_t* p, float a, float b, float c, float d) {
        half4 h;
        h[0] = (half_t)a; h[1] = (half_t)b; h[2] = (half_t)c; h[3] = (half_t)d;
        *reinterpret_cast<half4*>(p) = h;
    }
    // 8 consecutive input elements as they come from memory (so that a fetch can be issued long
    // before its first use), and their widening to float
    typedef u32x4 Raw8;
    static __device__ __forceinline__ Raw8 load_raw(const In* p) { return *reinterpret_cast<const u32x4*>(p); }
    static __device__ __forceinline__ Raw8 zero_raw() { return Raw8{0u, 0u, 0u, 0u}; }
    static __device__ __forceinline__ void unpack(const Raw8& raw, float out[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(raw[i] << 16);
            out[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ float widen(In x) { return __uint_as_float((uint32_t)x << 16); }
    // U~ travels in E: a 32x32 accumulator tile as UT_PIECES 16-byte pieces per lane, piece p = registers
    // UT_REGS p .. UT_REGS p + UT_REGS - 1 (its rounding is of the size of the operand rounding of U itself)
    typedef half8 UtVec;
    static constexpr int UT_PIECES = 2, UT_REGS = 8;
    static __device__ __forceinline__ UtVec ut_pack(const f32x16& acc, int p) { return from_acc(acc, p); }
    static __device__ __forceinline__ void ut_unpack(const UtVec& x, f32x16& acc, int p) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[8 * p + e] = (float)x[e];
    }
    // hardware exp2/log2 based: relative error ~1e-6 |x|, far inside the fp16 operand rounding
    static __device__ __forceinline__ float exp_(float x) { return __expf(x); }
    static __device__ __forceinline__ float log_(float x) { return __logf(x); }
};

template <> struct Elem<float> {
    typedef float In;
    typedef float Frag;
    static constexpr int PAD = 1;
    static constexpr int KSTEP = 2;
    static constexpr int STEPS_PER_TILE = 16;

    static __device__ __forceinline__ int slot4(int c) { return c; }
    static __device__ __forceinline__ Frag load(const float* row, int s, int g) {
        const int w = s & 15;
        return row[32 * (s >> 4) + 8 * (w >> 2) + 4 * g + (w & 3)];
    }
    static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ Frag scale(Frag f, const float* vec, int s, int g) {
        const int w = s & 15;
        return f * vec[32 * (s >> 4) + 8 * (w >> 2) + 4 * g + (w & 3)];
    }
    static __device__ __forceinline__ Frag from_acc(const f32x16& acc, int sub) { return acc[sub]; }
    static __device__ __forceinline__ Frag load_scaled(const float* x, const float* vec, int s, int g) {
        const int w = s & 15;
        const int c = 32 * (s >> 4) + 8 * (w >> 2) + 4 * g + (w & 3);
        return x[c] * vec[c];
    }
    static __device__ __forceinline__ void store4(float* p, float a, float b, float c, float d) {
        p[0] = a; p[1] = b; p[2] = c; p[3] = d;
    }
    struct Raw8 { f32x4 a, b; };
    static __device__ __forceinline__ Raw8 load_raw(const In* p) {
        return Raw8{*reinterpret_cast<const f32x4*>(p), *reinterpret_cast<const f32x4*>(p + 4)};
    }
    static __device__ __forceinline__ Raw8 zero_raw() { return Raw8{f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}}; }
    static __device__ __forceinline__ void unpack(const Raw8& raw, float out[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { out[i] = raw.a[i]; out[4 + i] = raw.b[i]; }
    }
    static __device__ __forceinline__ float widen(In x) { return x; }
    typedef f32x4 UtVec;
    static constexpr int UT_PIECES = 4, UT_REGS = 4;
    static __device__ __forceinline__ UtVec ut_pack(const f32x16& acc, int p) {
        return UtVec{acc[4 * p], acc[4 * p + 1], acc[4 * p + 2], acc[4 * p + 3]};
    }
    static __device__ __forceinline__ void ut_unpack(const UtVec& x, f32x16& acc, int p) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[4 * p + e] = x[e];
    }
    static __device__ __forceinline__ float exp_(float x) { return expf(x); }
    static __device__ __forceinline__ float log_(float x) { return logf(x); }
};

// Words that follow gam[64], dec[64] in a unit's aux block (int32).
enum { AUX_EMIT_SLOT = 0, AUX_TOK0 = 1, AUX_LEN = 2 };

// Byte layout of one (chunk, layer, value head) unit of the workspace.
//
// The chunk operands the recurrence kernel multiplies from the left (W, Q, K^T, P) are stored
// "fragment-major": fragment f of an operand is the 64-lane vector of MFMA A operands of one
// step, at [f][lane], so a wave fetches a step's operand with one fully coalesced vector load
// (from global memory, or from an LDS copy of the image without bank conflicts).  Fragment
// numbering: (row tile rt, step s) -> rt * steps + s, a row tile being 32 rows of the operand.
// The first STAGED_BYTES are what the recurrence kernel may copy to LDS in one linear pass;
// the accumulator-ordered U~ follows.
template <typename E, int DK, int DV> struct UnitLayout {
    static constexpr int C = 64;
    typedef typename Elem<E>::Frag Frag;
    static constexpr int FRAG_BYTES = 64 * (int)sizeof(Frag);            // one step of one wave
    static constexpr int NKD = DK / Elem<E>::KSTEP;                       // steps over d_k
    static constexpr int NKC = C / Elem<E>::KSTEP;                        // steps over the chunk's tokens
    static constexpr int W_BYTES = 2 * NKD * FRAG_BYTES;                  // W   [C][DK]: 2 row tiles x NKD
    static constexpr int KT_BYTES = (DK / 32) * NKC * FRAG_BYTES;         // K^T diag(dec) [DK][C]: DK/32 row tiles x NKC
    static constexpr int AUX_BYTES = 1024;                                // gam[C], dec[C] floats, bookkeeping words, padded
    static constexpr int Q_BYTES = 2 * NKD * FRAG_BYTES;                  // Q   [C][DK]: 2 row tiles x NKD
    static constexpr int P_BYTES = 2 * NKC * FRAG_BYTES;                  // P   [C][C]:  2 row tiles x NKC
    // what the state-dependent chain needs first (W, K^T, scale factors) is one contiguous run
    static constexpr int W_OFF = 0;
    static constexpr int KT_OFF = W_OFF + W_BYTES;
    static constexpr int AUX_OFF = KT_OFF + KT_BYTES;
    static constexpr int CHAIN_BYTES = AUX_OFF + AUX_BYTES;
    static constexpr int Q_OFF = CHAIN_BYTES;
    static constexpr int P_OFF = Q_OFF + Q_BYTES;
    static constexpr int STAGED_BYTES = P_OFF + P_BYTES;
    static constexpr int UT_OFF = STAGED_BYTES;                           // U~ in accumulator order, element type E
    static constexpr int UT_SLICE_BYTES = 2 * Elem<E>::UT_PIECES * 64 * (int)sizeof(typename Elem<E>::UtVec);   // one 32-column slice
    static constexpr int UNIT_BYTES = UT_OFF + (DV / 32) * UT_SLICE_BYTES;
    static_assert(CHAIN_BYTES % 1024 == 0 && UT_OFF % 1024 == 0, "1 KiB pieces for wave-wide 16-byte copies");
    static_assert(STAGED_BYTES % 16 == 0 && UNIT_BYTES % 256 == 0, "vector-copy granularity");
};

}  // namespace gdn
