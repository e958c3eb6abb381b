// Recurrence kernels: the state-dependent part, sequential over the chunks of one chain
// (request, layer, value head).  Each wave owns a 32-column slice of d_v for the whole chain:
// the slice of the state (as S^T, d_k x 32, fp32 accumulators), of U and of O.  Rows of the
// state are independent given the chunk's W, Q, K^T and P, so slices never exchange data.
//
// Per chunk, with S the state at the chunk start (all products on the matrix cores, the
// chunk operands read as ready-made fragments, the state-derived operands fed from
// registers):
//     U   = U~ + W S^T                        [C][32]
//     O^T = (S Q^T) diag(gam) + U^T P^T       [32][C]   (scale already folded into P)
//     S^T <- gam_C S^T + K^T-contraction:     S^T[d_k][d_v] += sum_j (dec_j K[j][d_k]) U[j][d_v]
// and, when the chunk ends at a checkpoint position, S is stored to its pool slot.
// A launch covers one slab (up to R consecutive chunks of every request); a chain that goes on
// in the next slab leaves its state in the carry buffer and picks it up there.
#pragma once
#include "gdn_mma.h"

namespace gdn {

struct RecurArgs {
    void* o;
    const char* ws_units;
    const int32_t* req_chunk_cu;
    const int32_t* req_src_slot;
    const int32_t* req_order;        // requests, longest chain first
    const float* state_src;
    float* state_dst;
    float* carry;                    // [request][L][H_v][d_v][d_k]: state handed from one slab to the next
    int64_t src_slot_stride, dst_slot_stride;
    int32_t slab_begin;              // first chunk round of this launch's slab
    int32_t R;                       // chunk rounds per slab
    int32_t L, H_qk, H_v;
    int64_t T_alloc;
    float scale;
    int32_t o_bf16;
};


// S^T tiles of one slice <-> the [d_v][d_k] fp32 state in a pool slot: register 4b+e of tile mt
// holds S[32 sl + lr][32 mt + 8b + 4g + e], i.e. 16-byte runs along d_k.
template <int MT>
__device__ __forceinline__ void load_state(f32x16 (&accS)[MT], const float* src, int g) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const f32x4 x = *reinterpret_cast<const f32x4*>(src + 32 * mt + 8 * b + 4 * g);
            accS[mt][4 * b] = x[0]; accS[mt][4 * b + 1] = x[1];
            accS[mt][4 * b + 2] = x[2]; accS[mt][4 * b + 3] = x[3];
        }
}
template <int MT>
__device__ __forceinline__ void store_state(const f32x16 (&accS)[MT], float* dst, int g) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const f32x4 x = {accS[mt][4 * b], accS[mt][4 * b + 1], accS[mt][4 * b + 2], accS[mt][4 * b + 3]};
            *reinterpret_cast<f32x4*>(dst + 32 * mt + 8 * b + 4 * g) = x;
        }
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// O is computed transposed, O^T[d_v][token] = S Q^T-contraction + U^T P^T-contraction, by swapping
// the operand roles (the state and U fragments are the left operands, the Q and P fragments the
// right ones; both fragment layouts are the same).  A lane then holds, for ONE token, runs of
// four consecutive d_v values, which go out as 16-byte (fp32) or 8-byte (bf16) stores, and the
// per-token factors gam_i and the "token < n" predicate are per-lane scalars.
// ot[tt]: tile of token tile tt (lane = token 32 tt + lr, register 4b+e = d_v 32 sl + 8b + 4g + e).
template <int DV, typename Args>
__device__ __forceinline__ void store_o_tile(const Args& a, int64_t row0, int hv, int sl, int lr, int g, int n,
                                             int tt, const f32x16& ot) {
    const int tok = 32 * tt + lr;
    if (tok < n) {
        const int64_t off = ((row0 + tok) * a.H_v + hv) * DV + 32 * sl + 4 * g;
        if (a.o_bf16) {
            uint16_t* p = reinterpret_cast<uint16_t*>(a.o) + off;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t lo = f32_to_bf16_rne(ot[4 * b]) | ((uint32_t)f32_to_bf16_rne(ot[4 * b + 1]) << 16);
                const uint32_t hi = f32_to_bf16_rne(ot[4 * b + 2]) | ((uint32_t)f32_to_bf16_rne(ot[4 * b + 3]) << 16);
                *reinterpret_cast<uint2*>(p + 8 * b) = make_uint2(lo, hi);
            }
        } else {
            float* p = reinterpret_cast<float*>(a.o) + off;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const f32x4 x = {ot[4 * b], ot[4 * b + 1], ot[4 * b + 2], ot[4 * b + 3]};
                *reinterpret_cast<f32x4*>(p + 8 * b) = x;
            }
        }
    }
}
template <int DV>
__device__ __forceinline__ void store_o_t(const RecurArgs& a, int64_t row0, int hv, int sl, int lr, int g, int n,
                                          const f32x16 (&ot)[2]) {
    store_o_tile<DV>(a, row0, hv, sl, lr, g, n, 0, ot[0]);
    store_o_tile<DV>(a, row0, hv, sl, lr, g, n, 1, ot[1]);
}

// Throughput variant.  The workgroup copies the unit's fragment image to LDS once per chunk and
// its NW waves (d_v slices) read fragments from there; the next image is prefetched into
// registers meanwhile.
template <typename E, int DK, int DV, int NW>
__global__ void __launch_bounds__(64 * NW) gdn_recur_kernel(RecurArgs a) {
    constexpr bool STAGED = true;
    typedef Elem<E> EL;
    typedef typename EL::Frag Frag;
    typedef UnitLayout<E, DK, DV> U;
    constexpr int C = 64;
    constexpr int NT = 64 * NW;
    constexpr int NS = DV / 32;              // slices per chain
    constexpr int SG = NS / NW;              // workgroups per chain
    constexpr int SPT = EL::STEPS_PER_TILE;
    constexpr int NKD = U::NKD;              // steps over d_k
    constexpr int NKC = U::NKC;              // steps over the chunk's tokens
    constexpr int MT = DK / 32;              // state tiles per slice
    static_assert(NS % NW == 0, "slices must split evenly over workgroups");

    extern __shared__ __align__(16) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: say so
    const int lr = lane & 31;
    const int g = lane >> 5;

    const int units = a.L * a.H_v;
    const int sg = blockIdx.x % SG;
    const int chain = blockIdx.x / SG;
    const int r = a.req_order[chain / units];
    const int lh = chain % units;
    const int l = lh / a.H_v;
    const int hv = lh % a.H_v;
    const int sl = sg * NW + wave;           // this wave's d_v slice
    const int c_last = a.req_chunk_cu[r + 1];
    const int c_begin = a.req_chunk_cu[r] + a.slab_begin;
    if (c_begin >= c_last) return;
    const int c_end = min(c_last, c_begin + a.R);

    // ---- start state: the pool slot (or zeros) in the first slab, the carried state afterwards
    f32x16 accS[MT];
    const int64_t head_off = ((int64_t)l * a.H_v + hv) * DV * DK + (int64_t)(32 * sl + lr) * DK;
    float* const carry = a.carry + (int64_t)r * units * DV * DK + head_off;
    {
        const int slot = a.req_src_slot[r];
        if (a.slab_begin > 0) {
            load_state<MT>(accS, carry, g);
        } else if (slot >= 0) {
            load_state<MT>(accS, a.state_src + slot * a.src_slot_stride + head_off, g);
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) accS[mt][i] = 0.f;
        }
    }

    const int64_t unit_stride = (int64_t)units * U::UNIT_BYTES;   // from one chunk to the next
    const char* unit = a.ws_units + ((int64_t)r * a.R * units + lh) * U::UNIT_BYTES;

    // image prefetch registers of the staged variant: NFULL vectors per thread plus a tail
    constexpr int NVEC = U::STAGED_BYTES / 16;
    constexpr int NFULL = STAGED ? NVEC / NT : 0;
    constexpr int TAIL = STAGED ? NVEC % NT : 0;
    u32x4 pre[NFULL > 0 ? NFULL : 1];
    u32x4 pre_tail = {0, 0, 0, 0};
#define GDN_PREFETCH_IMAGE(ptr)                                                   \
    {                                                                             \
        const u32x4* src_ = reinterpret_cast<const u32x4*>(ptr) + tid;            \
        _Pragma("unroll") for (int i_ = 0; i_ < NFULL; ++i_) pre[i_] = src_[i_ * NT]; \
        if (TAIL > 0 && tid < TAIL) pre_tail = src_[NFULL * NT];                  \
    }
    if (STAGED) GDN_PREFETCH_IMAGE(unit)
    // U~ of this wave's slice travels outside the staged image; it is fetched one chunk ahead as well, so
    // that no global load sits at the head of a chunk's dependent chain
    typedef typename EL::UtVec UtVec;
    constexpr int NUT = 2 * EL::UT_PIECES;
    UtVec ut_pre[NUT];
#define GDN_PREFETCH_UT(ptr)                                                                     \
    {                                                                                            \
        const UtVec* ut_ = reinterpret_cast<const UtVec*>((ptr) + U::UT_OFF) + (sl * NUT) * 64 + lane; \
        _Pragma("unroll") for (int k_ = 0; k_ < NUT; ++k_) ut_pre[k_] = ut_[k_ * 64];           \
    }
    GDN_PREFETCH_UT(unit)

    for (int c = c_begin; c < c_end; ++c, unit += unit_stride) {

        const char* img;
        {
            __syncthreads();  // the previous chunk's image is no longer read
            u32x4* dst = reinterpret_cast<u32x4*>(smem) + tid;
#pragma unroll
            for (int i = 0; i < NFULL; ++i) dst[i * NT] = pre[i];
            if (TAIL > 0 && tid < TAIL) dst[NFULL * NT] = pre_tail;
            __syncthreads();
            // (the last chunk re-reads its own image: no branch around the register loads)
            GDN_PREFETCH_IMAGE((c + 1 < c_end) ? unit + unit_stride : unit)
            img = smem;
        }
        const Frag* w_img = reinterpret_cast<const Frag*>(img + U::W_OFF) + lane;
        const Frag* q_img = reinterpret_cast<const Frag*>(img + U::Q_OFF) + lane;
        const Frag* kt_img = reinterpret_cast<const Frag*>(img + U::KT_OFF) + lane;
        const Frag* p_img = reinterpret_cast<const Frag*>(img + U::P_OFF) + lane;
        const float* gamS = reinterpret_cast<const float*>(img + U::AUX_OFF);
        const int32_t* meta = reinterpret_cast<const int32_t*>(gamS + 2 * C);
        const int eslot = meta[AUX_EMIT_SLOT];
        const int n = meta[AUX_LEN];
        const int64_t row0 = (int64_t)l * a.T_alloc + meta[AUX_TOK0];

        // U~ (this slice), already in accumulator order; then the next chunk's is requested
        f32x16 accU[2];
#pragma unroll
        for (int k = 0; k < NUT; ++k) EL::ut_unpack(ut_pre[k], accU[k / EL::UT_PIECES], k % EL::UT_PIECES);
        GDN_PREFETCH_UT((c + 1 < c_end) ? unit + unit_stride : unit)

        // state as the B operand of the two products that contract over d_k
        Frag sf[NKD];
#pragma unroll
        for (int s = 0; s < NKD; ++s) sf[s] = EL::from_acc(accS[s / SPT], s % SPT);

        // U = U~ + W S^T
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int s = 0; s < NKD; ++s) accU[rt] = EL::mma(w_img[(rt * NKD + s) * 64], sf[s], accU[rt]);

        // U as the register operand of both O += P U and the state update
        Frag uf[2 * SPT];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int s = 0; s < SPT; ++s) uf[rt * SPT + s] = EL::from_acc(accU[rt], s);

        // state update: S^T = gam_C S^T + sum_j (dec_j K^T[.][j]) U[j][.]
        const float gam_last = gamS[C - 1];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int i = 0; i < 16; ++i) accS[mt][i] *= gam_last;
#pragma unroll
            for (int s = 0; s < NKC; ++s) accS[mt] = EL::mma(kt_img[(mt * NKC + s) * 64], uf[s], accS[mt]);
        }

        // checkpoint emission: exact state after the last token of this chunk
        if (eslot >= 0) store_state<MT>(accS, a.state_dst + eslot * a.dst_slot_stride + head_off, g);

        // O^T = (S Q^T) diag(gam) + U^T P^T with the state of the chunk start (sf), off the chain
        f32x16 ot[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            f32x16 acc = {0};
#pragma unroll
            for (int s = 0; s < NKD; ++s) acc = EL::mma(sf[s], q_img[(tt * NKD + s) * 64], acc);
            const float gm = gamS[32 * tt + lr] * a.scale;
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[k] *= gm;
            // P is lower triangular: token tile 0 only sees key tile 0
#pragma unroll
            for (int s = 0; s < (tt + 1) * SPT; ++s) acc = EL::mma(uf[s], p_img[(tt * NKC + s) * 64], acc);
            ot[tt] = acc;
        }
        store_o_t<DV>(a, row0, hv, sl, lr, g, n, ot);
    }
    if (c_end < c_last) store_state<MT>(accS, carry, g);
}

#undef GDN_PREFETCH_IMAGE
#undef GDN_PREFETCH_UT

// s_waitcnt vmcnt(N) (gfx9 encoding: vmcnt in bits 3:0 and 15:14; other counters left alone)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(((N & 0x30) << 10) | (N & 0xF) | 0x0F70);
}

// Ring variant, for calls with at most one such workgroup per compute unit: NSW value-head slices of a
// chain per workgroup, one computing wave per slice and one more wave that only loads.  The operand image
// of a chunk and the U~ slices of this workgroup are copied into one of two LDS stages with 16-byte
// global->LDS loads (no registers) while the computing waves work on the other stage, so no global load
// sits on a chunk's dependent chain.  One barrier per chunk: the computing waves reach it when every LDS
// read of their stage has returned, the loader when the next chunk has landed.
template <typename E, int DK, int DV, int NSW>
struct RingSmem {
    typedef UnitLayout<E, DK, DV> U;
    static constexpr int IMG_PIECES = U::STAGED_BYTES / 1024;                  // whole 1 KiB pieces of the image
    static constexpr int IMG_TAIL_LANES = (U::STAGED_BYTES % 1024) / 16;      // lanes of its last, partial piece
    static constexpr int UT_PIECES = NSW * U::UT_SLICE_BYTES / 1024;
    static constexpr int UT_OFF = (U::STAGED_BYTES + 1023) / 1024 * 1024;     // U~ slices behind the image
    static constexpr int STAGE_BYTES = UT_OFF + NSW * U::UT_SLICE_BYTES;
    static constexpr int BYTES = 2 * STAGE_BYTES;
    static_assert(BYTES <= 160 * 1024, "LDS");
    static_assert((NSW * U::UT_SLICE_BYTES) % 1024 == 0 && U::STAGED_BYTES % 16 == 0, "piece sizes");
};

template <typename E, int DK, int DV, int NSW>
__device__ __forceinline__ void recur_ring_body(const RecurArgs& a, const int block) {
    typedef Elem<E> EL;
    typedef typename EL::Frag Frag;
    typedef typename EL::UtVec UtVec;
    typedef UnitLayout<E, DK, DV> U;
    typedef RingSmem<E, DK, DV, NSW> SM;
    constexpr int C = 64;
    constexpr int NS = DV / 32;
    constexpr int SG = NS / NSW;             // workgroups per chain
    constexpr int SPT = EL::STEPS_PER_TILE;
    constexpr int NKD = U::NKD;
    constexpr int NKC = U::NKC;
    constexpr int MT = DK / 32;
    constexpr int NUT = 2 * EL::UT_PIECES;

    extern __shared__ __align__(16) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: say so
    const int lr = lane & 31;
    const int g = lane >> 5;

    const int units = a.L * a.H_v;
    const int sg = block % SG;
    const int chain = block / SG;
    const int r = a.req_order[chain / units];
    const int lh = chain % units;
    const int l = lh / a.H_v;
    const int hv = lh % a.H_v;
    const int c_last = a.req_chunk_cu[r + 1];
    const int c_begin = a.req_chunk_cu[r] + a.slab_begin;
    if (c_begin >= c_last) return;
    const int n_chunks = min(c_last - c_begin, a.R);
    const int64_t unit_stride = (int64_t)units * U::UNIT_BYTES;
    const char* unit0 = a.ws_units + ((int64_t)r * a.R * units + lh) * U::UNIT_BYTES;

    if (wave == NSW) {
        // ------------------------------------------------------------ loader wave
        // A chunk is more pieces than the 6-bit outstanding-load counter should hold at once: it is
        // issued in two parts with a wait in between.
        constexpr int NP = SM::IMG_PIECES;
        constexpr int NA = NP > 40 ? 40 : NP, NB = NP - NA;
        static_assert(16 + NB + 1 + SM::UT_PIECES <= 63 && NA <= 63, "parts vs the outstanding-load counter");
        auto issue = [&](int i) {
            const char* src = unit0 + i * unit_stride + lane * 16;
            char* dst = smem + (i & 1) * SM::STAGE_BYTES;
#pragma unroll
            for (int k = 0; k < NA; ++k)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + k * 1024),
                                                 (__attribute__((address_space(3))) void*)(dst + k * 1024), 16, 0, 0);
            if (NB > 0) wait_vmcnt<16>();
#pragma unroll
            for (int k = NA; k < NP; ++k)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + k * 1024),
                                                 (__attribute__((address_space(3))) void*)(dst + k * 1024), 16, 0, 0);
            if (SM::IMG_TAIL_LANES > 0 && lane < SM::IMG_TAIL_LANES)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + NP * 1024),
                                                 (__attribute__((address_space(3))) void*)(dst + NP * 1024), 16, 0, 0);
            const char* usrc = src + U::UT_OFF + (sg * NSW) * U::UT_SLICE_BYTES;
#pragma unroll
            for (int k = 0; k < SM::UT_PIECES; ++k)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(usrc + k * 1024),
                                                 (__attribute__((address_space(3))) void*)(dst + SM::UT_OFF + k * 1024), 16, 0, 0);
        };
        issue(0);
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();               // chunk 0 is in stage 0
        for (int i = 0; i < n_chunks; ++i) {
            if (i + 1 < n_chunks) issue(i + 1);     // into the stage the computing waves left at the last barrier
            wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();           // chunk i is consumed, chunk i + 1 has landed
        }
        return;
    }

    // ---------------------------------------------------------------- computing waves
    const int sl = sg * NSW + wave;          // this wave's d_v slice
    f32x16 accS[MT];
    const int64_t head_off = ((int64_t)l * a.H_v + hv) * DV * DK + (int64_t)(32 * sl + lr) * DK;
    float* const carry = a.carry + (int64_t)r * units * DV * DK + head_off;
    {
        const int slot = a.req_src_slot[r];
        if (a.slab_begin > 0) {
            load_state<MT>(accS, carry, g);
        } else if (slot >= 0) {
            load_state<MT>(accS, a.state_src + slot * a.src_slot_stride + head_off, g);
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) accS[mt][i] = 0.f;
        }
    }
    __syncthreads();   // chunk 0 is in stage 0
    for (int i = 0; i < n_chunks; ++i) {
        const char* img = smem + (i & 1) * SM::STAGE_BYTES;
        const Frag* w_img = reinterpret_cast<const Frag*>(img + U::W_OFF) + lane;
        const Frag* q_img = reinterpret_cast<const Frag*>(img + U::Q_OFF) + lane;
        const Frag* kt_img = reinterpret_cast<const Frag*>(img + U::KT_OFF) + lane;
        const Frag* p_img = reinterpret_cast<const Frag*>(img + U::P_OFF) + lane;
        const UtVec* ut = reinterpret_cast<const UtVec*>(img + SM::UT_OFF) + (wave * NUT) * 64 + lane;
        const float* gamS = reinterpret_cast<const float*>(img + U::AUX_OFF);
        const int32_t* meta = reinterpret_cast<const int32_t*>(gamS + 2 * C);
        const int eslot = meta[AUX_EMIT_SLOT];
        const int n = meta[AUX_LEN];
        const int64_t row0 = (int64_t)l * a.T_alloc + meta[AUX_TOK0];

        f32x16 accU[2];
#pragma unroll
        for (int k = 0; k < NUT; ++k) EL::ut_unpack(ut[k * 64], accU[k / EL::UT_PIECES], k % EL::UT_PIECES);
        Frag sf[NKD];
#pragma unroll
        for (int s = 0; s < NKD; ++s) sf[s] = EL::from_acc(accS[s / SPT], s % SPT);
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int s = 0; s < NKD; ++s) accU[rt] = EL::mma(w_img[(rt * NKD + s) * 64], sf[s], accU[rt]);
        Frag uf[2 * SPT];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int s = 0; s < SPT; ++s) uf[rt * SPT + s] = EL::from_acc(accU[rt], s);
        const float gam_last = gamS[C - 1];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int k = 0; k < 16; ++k) accS[mt][k] *= gam_last;
#pragma unroll
            for (int s = 0; s < NKC; ++s) accS[mt] = EL::mma(kt_img[(mt * NKC + s) * 64], uf[s], accS[mt]);
        }
        if (eslot >= 0) store_state<MT>(accS, a.state_dst + eslot * a.dst_slot_stride + head_off, g);
        f32x16 ot[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            f32x16 acc = {0};
#pragma unroll
            for (int s = 0; s < NKD; ++s) acc = EL::mma(sf[s], q_img[(tt * NKD + s) * 64], acc);
            const float gm = gamS[32 * tt + lr] * a.scale;
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[k] *= gm;
#pragma unroll
            for (int s = 0; s < (tt + 1) * SPT; ++s) acc = EL::mma(uf[s], p_img[(tt * NKC + s) * 64], acc);
            ot[tt] = acc;
        }
        store_o_t<DV>(a, row0, hv, sl, lr, g, n, ot);
        // Done with this stage once every LDS read has returned; the stores of O stay in flight across
        // the barrier (waiting for them here would put a memory round trip on every chunk).
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only
        __builtin_amdgcn_s_barrier();         // the next chunk has landed in the other stage
    }
    if (c_begin + n_chunks < c_last) store_state<MT>(accS, carry, g);
}

template <typename E, int DK, int DV, int NSW>
__global__ void __launch_bounds__(64 * (NSW + 1)) gdn_recur_ring_kernel(RecurArgs a) {
    recur_ring_body<E, DK, DV, NSW>(a, (int)blockIdx.x);
}

template <typename E, int DK, int DV>
constexpr int recur_smem_bytes() {
    return UnitLayout<E, DK, DV>::STAGED_BYTES;
}

// Latency variant, for calls with too few chains to fill the chip: the per-chunk dependent
// chain bounds the run time, so everything else is taken off it.  One workgroup per
// (chain, d_v slice) with four waves, one per SIMD:
//   wave 0 ("chain")      keeps the state and runs only the dependent part, U = U~ + W S^T and
//                         the state update, reading W, K^T, U~ and the scale factors from an LDS
//                         ring; its matrix instructions issue back to back, conversions, the
//                         decay of the state and LDS traffic ride in their shadow;
//   waves 1, 2 ("output") compute O one chunk behind, one token tile each, from the state and U
//                         fragments wave 0 leaves in LDS (double buffered), with Q and P fetched
//                         from global memory into registers three chunks ahead;
//   wave 3 ("loader")     fills the ring two chunks ahead with 16-byte global->LDS loads (lane l
//                         of an instruction lands at base + 16 l, so 1 KiB of the fragment-major
//                         image per instruction, no registers).
// Ring stage s holds chunk i with i % 3 == s.  Every wave passes one barrier before the first
// chunk and one per chunk.  The chain wave reaches chunk i's barrier once it has read all it
// needs of chunk i's stage and has published chunk i's fragments; the loader reaches it only
// when chunk i+1 has landed, and refills the released stage with chunk i+3 right after it.
template <typename E, int DK, int DV>
struct QuadSmem {
    typedef UnitLayout<E, DK, DV> U;
    static constexpr int STAGES = 3;
    static constexpr int UT_OFF = U::CHAIN_BYTES;                     // stage: [W | K^T | aux | U~ slice]
    static constexpr int STAGE_BYTES = U::CHAIN_BYTES + U::UT_SLICE_BYTES;
    static constexpr int XCH_OFF = STAGES * STAGE_BYTES;
    static constexpr int XCH_FRAGS = U::NKD + U::NKC;                 // state fragments, then U fragments
    static constexpr int BYTES = XCH_OFF + 2 * XCH_FRAGS * U::FRAG_BYTES;
    static constexpr int DMA_PER_STAGE = STAGE_BYTES / 1024;
    static_assert(BYTES <= 160 * 1024, "LDS");
};

#define GDN_FENCE() __builtin_amdgcn_sched_barrier(0)   // nothing is scheduled across this point

// The work of one latency-variant workgroup: workgroup `wg` of the `nb` that cover the chains' slices.
template <typename E, int DK, int DV>
__device__ __forceinline__ void recur_quad_body(const RecurArgs& a, const int wg, const int nb) {
    typedef Elem<E> EL;
    typedef typename EL::Frag Frag;
    typedef UnitLayout<E, DK, DV> U;
    typedef QuadSmem<E, DK, DV> SM;
    constexpr int C = 64;
    constexpr int NS = DV / 32;
    constexpr int SPT = EL::STEPS_PER_TILE;
    constexpr int NKD = U::NKD;
    constexpr int NKC = U::NKC;
    constexpr int MT = DK / 32;
    typedef typename EL::UtVec UtVec;
    constexpr int NUT = 2 * EL::UT_PIECES;   // 16-byte pieces of a slice's U~ per lane

    extern __shared__ __align__(16) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: say so
    const int lr = lane & 31;
    const int g = lane >> 5;

    // Workgroups are handed to the eight XCDs round robin, and each XCD has its own L2.  The NS
    // slices of a chain read the same W, K^T, Q and P, so consecutive work items are given to
    // workgroups of the same XCD: item = (position of this XCD's first workgroup in a by-XCD
    // ordering) + (index of this workgroup within its XCD).
    int item;
    {
        const int x = wg & 7, q = nb >> 3, rem = nb & 7;
        item = (x < rem ? x * (q + 1) : rem * (q + 1) + (x - rem) * q) + (wg >> 3);
    }
    const int units = a.L * a.H_v;
    const int sl = item % NS;
    const int chain = item / NS;
    const int r = a.req_order[chain / units];
    const int lh = chain % units;
    const int l = lh / a.H_v;
    const int hv = lh % a.H_v;
    const int c_last = a.req_chunk_cu[r + 1];
    const int c_begin = a.req_chunk_cu[r] + a.slab_begin;
    if (c_begin >= c_last) return;
    const int n_chunks = min(c_last - c_begin, a.R);

    const int64_t unit_stride = (int64_t)units * U::UNIT_BYTES;
    const char* unit0 = a.ws_units + ((int64_t)r * a.R * units + lh) * U::UNIT_BYTES;

    if (wave == 3) {
        // ------------------------------------------------------------ loader wave
        // Two stages' loads are in flight in steady state, more than the 6-bit outstanding-load
        // counter holds, so a stage is issued in two parts with a wait in between that keeps
        // the count at 63 or below.
        constexpr int NP = SM::DMA_PER_STAGE;
        constexpr int NA = 2 * NP <= 63 ? NP : 63 - NP, NB = NP - NA;   // first part, second part
        constexpr int NCHAIN = U::CHAIN_BYTES / 1024;
        static_assert(NP <= 62 && NA > 0 && NB >= 0, "stage size vs outstanding-load counter");
        auto issue = [&](int i, int stage, int k0, int k1) {
            const int ii = i < n_chunks ? i : n_chunks - 1;   // past the end: harmless re-read
            const char* u = unit0 + ii * unit_stride;
            const char* g_chain = u + lane * 16;
            const char* g_ut = u + U::UT_OFF + sl * U::UT_SLICE_BYTES + lane * 16;
            char* dst = smem + stage * SM::STAGE_BYTES;
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                if (k < k0 || k >= k1) continue;
                const char* src = k < NCHAIN ? g_chain + k * 1024 : g_ut + (k - NCHAIN) * 1024;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                                 (__attribute__((address_space(3))) void*)(dst + k * 1024), 16, 0, 0);
            }
        };
        // issue_stage: with at most NP loads outstanding on entry, at most 63 at any time
        auto issue_stage = [&](int i, int stage) {
            issue(i, stage, 0, NA);
            if (NB > 0) {
                wait_vmcnt<63 - NB>();
                issue(i, stage, NA, NP);
            }
        };
        issue(0, 0, 0, NP);
        issue_stage(1, 1);
        wait_vmcnt<NP>();                       // chunk 0 has landed
        issue_stage(2, 2);
        __builtin_amdgcn_s_barrier();
        int stage = 0;
        for (int i = 0; i < n_chunks; ++i) {
            wait_vmcnt<NP>();                   // chunk i+1 has landed (chunk i+2 may be in flight)
            __builtin_amdgcn_s_barrier();       // the chain wave is done with chunk i's stage
            issue_stage(i + 3, stage);
            stage = stage == 2 ? 0 : stage + 1;
        }
        wait_vmcnt<0>();
    } else if (wave == 0) {
        // ------------------------------------------------------------ chain wave
        f32x16 accS[MT];
        const int64_t head_off = ((int64_t)l * a.H_v + hv) * DV * DK + (int64_t)(32 * sl + lr) * DK;
        float* const carry = a.carry + (int64_t)r * units * DV * DK + head_off;
        {
            const int slot = a.req_src_slot[r];
            if (a.slab_begin > 0) {
                load_state<MT>(accS, carry, g);
            } else if (slot >= 0) {
                load_state<MT>(accS, a.state_src + slot * a.src_slot_stride + head_off, g);
            } else {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) accS[mt][i] = 0.f;
            }
        }
        __syncthreads();   // chunk 0 is in the ring
        Frag* const xch0 = reinterpret_cast<Frag*>(smem + SM::XCH_OFF) + lane;
        // W fragments and U~ accumulators of the chunk about to be processed
        Frag wf[2 * NKD];
        f32x16 accU[2];
        {
            const Frag* w_ = reinterpret_cast<const Frag*>(smem + U::W_OFF) + lane;
            const UtVec* ut_ = reinterpret_cast<const UtVec*>(smem + SM::UT_OFF) + lane;
#pragma unroll
            for (int k = 0; k < 2 * NKD; ++k) wf[k] = w_[k * 64];
#pragma unroll
            for (int k = 0; k < NUT; ++k) EL::ut_unpack(ut_[k * 64], accU[k / EL::UT_PIECES], k % EL::UT_PIECES);
        }
        int stage = 0;
        for (int i = 0; i < n_chunks; ++i) {
            const char* st = smem + stage * SM::STAGE_BYTES;
            stage = stage == 2 ? 0 : stage + 1;
            const char* st_next = smem + stage * SM::STAGE_BYTES;
            const Frag* kt_img = reinterpret_cast<const Frag*>(st + U::KT_OFF) + lane;
            const float* gamS = reinterpret_cast<const float*>(st + U::AUX_OFF);
            Frag* xch = xch0 + (i & 1) * SM::XCH_FRAGS * 64;
            const float gam_last = gamS[C - 1];
            const int eslot = reinterpret_cast<const int32_t*>(gamS + 2 * C)[AUX_EMIT_SLOT];

            // Everything below is laid out as short groups, one matrix instruction plus what is
            // meant to execute in its shadow, separated by scheduling fences.  The vector work
            // (conversions, the decay of the state) is spread so that no group carries more than
            // six such instructions.
            Frag sf[NKD], kf[MT * NKC], uf[NKC];
            auto decay = [&](int mt, int r0, int r1) {
#pragma unroll
                for (int e = r0; e < r1; ++e) {
                    float x = accS[mt][e] * gam_last;
                    pin(x);
                    accS[mt][e] = x;
                }
            };
            sf[0] = EL::from_acc(accS[0], 0);
            pin(sf[0]);
            GDN_FENCE();
            // ---- U token tile 0: state -> B fragments just ahead of their use, published to the
            //      output waves; decay of the first state tile (its fragments were taken first)
#pragma unroll
            for (int k = 0; k < NKD; ++k) {
                accU[0] = EL::mma(wf[k], sf[k], accU[0]);
                if (k + 1 < NKD) {
                    sf[k + 1] = EL::from_acc(accS[(k + 1) / SPT], (k + 1) % SPT);
                    pin(sf[k + 1]);
                }
                xch[k * 64] = sf[k];
                decay(0, k * (16 / NKD), (k + 1) * (16 / NKD));
                GDN_FENCE();
            }
            // ---- U token tile 1: decay of the second state tile; K^T fragments are read;
            //      tile 0 of U is converted as soon as its last product has drained
#pragma unroll
            for (int k = 0; k < NKD; ++k) {
                accU[1] = EL::mma(wf[NKD + k], sf[k], accU[1]);
                decay(1, k * (16 / NKD), (k + 1) * (16 / NKD));
#pragma unroll
                for (int j = 0; j < (MT * NKC) / NKD; ++j) kf[k * ((MT * NKC) / NKD) + j] = kt_img[(k * ((MT * NKC) / NKD) + j) * 64];
                // conversion piece p of tile 0 at step 2 + p * stride (late enough for the data)
                constexpr int stride = (NKD - 2) / SPT > 0 ? (NKD - 2) / SPT : 1;
                if (k >= 2 && (k - 2) % stride == 0 && (k - 2) / stride < SPT) {
                    const int p = (k - 2) / stride;
                    uf[p] = EL::from_acc(accU[0], p);
                    pin(uf[p]);
                    xch[(NKD + p) * 64] = uf[p];
                }
                GDN_FENCE();
            }
            // (steps of tile 0's conversion that did not fit into the loop above)
            {
                constexpr int stride = (NKD - 2) / SPT > 0 ? (NKD - 2) / SPT : 1;
                constexpr int done = (NKD - 2 + stride - 1) / stride < SPT ? ((NKD - 2 + stride - 1) / stride > 0 ? (NKD - 2 + stride - 1) / stride : 0) : SPT;
#pragma unroll
                for (int p = done; p < SPT; ++p) {
                    uf[p] = EL::from_acc(accU[0], p);
                    pin(uf[p]);
                    xch[(NKD + p) * 64] = uf[p];
                }
                GDN_FENCE();
            }
            // ---- state update, one state tile after the other (all token steps of a tile back
            //      to back).  First half of the tiles: tile 1 of U is converted under the first
            //      products, the state tiles two further on are decayed.
#pragma unroll
            for (int mt = 0; mt < MT / 2; ++mt) {
#pragma unroll
                for (int s = 0; s < NKC; ++s) {
                    accS[mt] = EL::mma(kf[mt * NKC + s], uf[s], accS[mt]);
                    if (mt == 0 && s < SPT) {
                        uf[SPT + s] = EL::from_acc(accU[1], s);
                        pin(uf[SPT + s]);
                        xch[(NKD + SPT + s) * 64] = uf[SPT + s];
                    }
                    if (mt + 2 < MT) decay(mt + 2, s * (16 / NKC), (s + 1) * (16 / NKC));
                    GDN_FENCE();
                }
            }
            __syncthreads();   // this chunk's fragments are published, its ring stage is released,
                               // the next chunk's stage has landed
            // ---- second half of the state tiles, the next chunk's W fragments and U~ being read
            //      in their shadow
            {
                const Frag* w_ = reinterpret_cast<const Frag*>(st_next + U::W_OFF) + lane;
                const UtVec* ut_ = reinterpret_cast<const UtVec*>(st_next + SM::UT_OFF) + lane;
                constexpr int NM = (MT - MT / 2) * NKC;           // matrix instructions left
                constexpr int WPM = (2 * NKD + NM - 1) / NM;      // W fragments read per instruction
                int m = 0;
#pragma unroll
                for (int mt = MT / 2; mt < MT; ++mt)
#pragma unroll
                    for (int s = 0; s < NKC; ++s, ++m) {
                        accS[mt] = EL::mma(kf[mt * NKC + s], uf[s], accS[mt]);
                        if (mt + 2 < MT) decay(mt + 2, s * (16 / NKC), (s + 1) * (16 / NKC));
#pragma unroll
                        for (int j = 0; j < WPM; ++j)
                            if (m * WPM + j < 2 * NKD) wf[m * WPM + j] = w_[(m * WPM + j) * 64];
                        if (m < NUT) EL::ut_unpack(ut_[m * 64], accU[m / EL::UT_PIECES], m % EL::UT_PIECES);
                        GDN_FENCE();
                    }
                // (U~ pieces beyond the number of matrix instructions)
#pragma unroll
                for (int k = NM; k < NUT; ++k) EL::ut_unpack(ut_[k * 64], accU[k / EL::UT_PIECES], k % EL::UT_PIECES);
            }
            // checkpoint emission: exact state after the last token of this chunk
            if (eslot >= 0) store_state<MT>(accS, a.state_dst + eslot * a.dst_slot_stride + head_off, g);
        }
        if (c_begin + n_chunks < c_last) store_state<MT>(accS, carry, g);
    } else {
        // ------------------------------------------------------------ output waves
        // Wave 1 owns token tile 0, wave 2 token tile 1.  Three register sets of Q/P fragments
        // rotate: the set a chunk has just used is refilled with the chunk three ahead, so a
        // load has three chunk times to arrive.
        const int tt = wave - 1;
        const int np = (tt + 1) * SPT;           // P is lower triangular: tile 0 only sees key tile 0
        Frag qf0[NKD], qf1[NKD], qf2[NKD], pf0[NKC], pf1[NKC], pf2[NKC];
        float gm0, gm1, gm2;
        int t00, t01, t02, n0, n1, n2;
        auto load_set = [&](int j, Frag (&qf)[NKD], Frag (&pf)[NKC], float& gm, int& tok0, int& nn) {
            const int jj = j < n_chunks ? j : n_chunks - 1;   // past the end: harmless re-read
            const char* u = unit0 + jj * unit_stride;
            const Frag* q_ = reinterpret_cast<const Frag*>(u + U::Q_OFF) + tt * NKD * 64 + lane;
            const Frag* p_ = reinterpret_cast<const Frag*>(u + U::P_OFF) + tt * NKC * 64 + lane;
            const float* g_ = reinterpret_cast<const float*>(u + U::AUX_OFF);
            const int32_t* m_ = reinterpret_cast<const int32_t*>(g_ + 2 * C);
#pragma unroll
            for (int k = 0; k < NKD; ++k) qf[k] = q_[k * 64];
#pragma unroll
            for (int k = 0; k < NKC; ++k)
                if (k < np) pf[k] = p_[k * 64];
            gm = g_[32 * tt + lr];
            tok0 = m_[AUX_TOK0];
            nn = m_[AUX_LEN];
        };
        auto step = [&](int j, Frag (&qf)[NKD], Frag (&pf)[NKC], float& gm, int& tok0, int& nn) {
            __syncthreads();   // the chain wave has left chunk j's state and U fragments
            const Frag* xch = reinterpret_cast<const Frag*>(smem + SM::XCH_OFF) + (j & 1) * SM::XCH_FRAGS * 64 + lane;
            Frag sf[NKD], uf[NKC];
#pragma unroll
            for (int k = 0; k < NKD; ++k) sf[k] = xch[k * 64];
#pragma unroll
            for (int k = 0; k < NKC; ++k)
                if (k < np) uf[k] = xch[(NKD + k) * 64];
            f32x16 acc = {0};
#pragma unroll
            for (int k = 0; k < NKD; ++k) acc = EL::mma(sf[k], qf[k], acc);
            const float sc = gm * a.scale;
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[k] *= sc;
#pragma unroll
            for (int k = 0; k < NKC; ++k)
                if (k < np) acc = EL::mma(uf[k], pf[k], acc);
            const int n = nn;
            const int64_t row0 = (int64_t)l * a.T_alloc + tok0;
            load_set(j + 3, qf, pf, gm, tok0, nn);   // refill the set just used
            store_o_tile<DV>(a, row0, hv, sl, lr, g, n, tt, acc);
        };
        load_set(0, qf0, pf0, gm0, t00, n0);
        load_set(1, qf1, pf1, gm1, t01, n1);
        load_set(2, qf2, pf2, gm2, t02, n2);
        __syncthreads();   // matches the barrier before the first chunk
        for (int i = 0; i < n_chunks; i += 3) {
            step(i, qf0, pf0, gm0, t00, n0);
            if (i + 1 < n_chunks) step(i + 1, qf1, pf1, gm1, t01, n1);
            if (i + 2 < n_chunks) step(i + 2, qf2, pf2, gm2, t02, n2);
        }
    }
}

#undef GDN_FENCE

template <typename E, int DK, int DV>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) gdn_recur_quad_kernel(RecurArgs a) {
    recur_quad_body<E, DK, DV>(a, (int)blockIdx.x, (int)gridDim.x);
}

}  // namespace gdn
