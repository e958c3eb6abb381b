// Recurrence kernel: the state-dependent part, sequential over the chunks of one chain
// (request, layer, value head).  Each wave owns a 32-column slice of d_v for the whole chain:
// the slice of the state (as S^T, d_k x 32, fp32 accumulators), of U and of O.  Rows of the
// state are independent given the chunk's W, Q, K^T and P, so waves never exchange data; a
// workgroup is NW waves (slices) of one chain sharing the staged tiles in LDS.
//
// Per chunk, with S the state at the chunk start (all products on the matrix cores, the
// left operands read as ready-made fragments, the state-derived right operands fed from
// registers):
//     U  = U~ + W S^T                      [C][32]
//     O  = diag(gam) (Q S^T) + P U         [C][32]   (scale already folded into gam, P)
//     S^T <- gam_C S^T + K^T-contraction:  S^T[d_k][d_v] += sum_j K[j][d_k] dec_j U[j][d_v]
// and, when the chunk ends at a checkpoint position, S is stored to its pool slot.
#pragma once
#include "gdn_mma.h"

namespace gdn {

struct RecurArgs {
    void* o;
    const char* ws_units;
    const int32_t* chunk_tok0;
    const int32_t* chunk_len;
    const int32_t* chunk_emit_slot;  // destination slot after the chunk, or -1
    const int32_t* req_chunk_cu;
    const int32_t* req_src_slot;
    const int32_t* req_order;        // requests, longest chain first
    const float* state_src;
    float* state_dst;
    int64_t src_slot_stride, dst_slot_stride;
    int32_t L, H_qk, H_v;
    int64_t T_alloc;
    float scale;
    int32_t o_bf16;
    int32_t debug_same_unit;  // timing experiment: every chunk reads the first unit (wrong results)
};

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
template <int DV>
__device__ __forceinline__ void store_o_t(const RecurArgs& a, int64_t row0, int hv, int sl, int lr, int g, int n,
                                          const f32x16 (&ot)[2]) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const int tok = 32 * tt + lr;
        if (tok < n) {
            const int64_t off = ((row0 + tok) * a.H_v + hv) * DV + 32 * sl + 4 * g;
            if (a.o_bf16) {
                uint16_t* p = reinterpret_cast<uint16_t*>(a.o) + off;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t lo = f32_to_bf16_rne(ot[tt][4 * b]) | ((uint32_t)f32_to_bf16_rne(ot[tt][4 * b + 1]) << 16);
                    const uint32_t hi = f32_to_bf16_rne(ot[tt][4 * b + 2]) | ((uint32_t)f32_to_bf16_rne(ot[tt][4 * b + 3]) << 16);
                    *reinterpret_cast<uint2*>(p + 8 * b) = make_uint2(lo, hi);
                }
            } else {
                float* p = reinterpret_cast<float*>(a.o) + off;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const f32x4 x = {ot[tt][4 * b], ot[tt][4 * b + 1], ot[tt][4 * b + 2], ot[tt][4 * b + 3]};
                    *reinterpret_cast<f32x4*>(p + 8 * b) = x;
                }
            }
        }
    }
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
    const int wave = tid >> 6;
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
    const int c_begin = a.req_chunk_cu[r], c_end = a.req_chunk_cu[r + 1];
    if (c_begin == c_end) return;

    // ---- start state: S^T tiles, register 4b+e of tile mt <-> S[32 sl + lr][32 mt + 8b + 4g + e]
    f32x16 accS[MT];
    const int64_t head_off = ((int64_t)l * a.H_v + hv) * DV * DK + (int64_t)(32 * sl + lr) * DK;
    {
        const int slot = a.req_src_slot[r];
        if (slot >= 0) {
            const float* src = a.state_src + slot * a.src_slot_stride + head_off;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const f32x4 x = *reinterpret_cast<const f32x4*>(src + 32 * mt + 8 * b + 4 * g);
                    accS[mt][4 * b] = x[0]; accS[mt][4 * b + 1] = x[1];
                    accS[mt][4 * b + 2] = x[2]; accS[mt][4 * b + 3] = x[3];
                }
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) accS[mt][i] = 0.f;
        }
    }

    const int64_t unit_stride = (int64_t)units * U::UNIT_BYTES;   // from one chunk to the next
    const char* unit = a.ws_units + ((int64_t)c_begin * units + lh) * U::UNIT_BYTES;

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

    for (int c = c_begin; c < c_end; ++c, unit += unit_stride) {
        const int tok0 = a.chunk_tok0[c];
        const int n = a.chunk_len[c];
        const int eslot = a.chunk_emit_slot[c];
        const int64_t row0 = (int64_t)l * a.T_alloc + tok0;

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
        const float* decS = gamS + C;

        // U~ (this slice), already in accumulator order
        f32x16 accU[2];
        {
            const f32x4* ut = reinterpret_cast<const f32x4*>(unit + U::UT_OFF);
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const f32x4 x = ut[((sl * 2 + rt) * 4 + b) * 64 + lane];
                    accU[rt][4 * b] = x[0]; accU[rt][4 * b + 1] = x[1];
                    accU[rt][4 * b + 2] = x[2]; accU[rt][4 * b + 3] = x[3];
                }
        }

        // state as the B operand of the two products that contract over d_k
        Frag sf[NKD];
#pragma unroll
        for (int s = 0; s < NKD; ++s) sf[s] = EL::from_acc(accS[s / SPT], s % SPT);

        // U = U~ + W S^T
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int s = 0; s < NKD; ++s) accU[rt] = EL::mma(w_img[(rt * NKD + s) * 64], sf[s], accU[rt]);

        // U as B operand: plain for O += P U, decayed to the chunk end for the state update
        Frag uf[2 * SPT], ud[2 * SPT];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            f32x16 d = accU[rt];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const f32x4 dc = *reinterpret_cast<const f32x4*>(decS + 32 * rt + 8 * b + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) d[4 * b + e] *= dc[e];
            }
#pragma unroll
            for (int s = 0; s < SPT; ++s) {
                uf[rt * SPT + s] = EL::from_acc(accU[rt], s);
                ud[rt * SPT + s] = EL::from_acc(d, s);
            }
        }

        // state update: S^T = gam_C S^T + sum_j K^T[.][j] (dec_j U[j][.])
        const float gam_last = gamS[C - 1];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int i = 0; i < 16; ++i) accS[mt][i] *= gam_last;
#pragma unroll
            for (int s = 0; s < NKC; ++s) accS[mt] = EL::mma(kt_img[(mt * NKC + s) * 64], ud[s], accS[mt]);
        }

        // checkpoint emission: exact state after the last token of this chunk
        if (eslot >= 0) {
            float* dst = a.state_dst + eslot * a.dst_slot_stride + head_off;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const f32x4 x = {accS[mt][4 * b], accS[mt][4 * b + 1], accS[mt][4 * b + 2], accS[mt][4 * b + 3]};
                    *reinterpret_cast<f32x4*>(dst + 32 * mt + 8 * b + 4 * g) = x;
                }
        }

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
}

#undef GDN_PREFETCH_IMAGE

template <typename E, int DK, int DV>
constexpr int recur_smem_bytes() {
    return UnitLayout<E, DK, DV>::STAGED_BYTES;
}

// Latency variant, for calls with too few chains to fill the chip: the per-chunk dependent
// chain bounds the run time, so it is cut to the minimum and memory latency is taken off it.
// One workgroup per (chain, d_v slice) with three waves:
//   wave 0 ("chain")  keeps the state and runs only the dependent part, U = U~ + W S^T and the
//                     state update, reading W, K^T, U~ and the scale factors from an LDS ring;
//   wave 1 ("output") computes O = diag(gam) Q S^T + P U one chunk behind, from the state and U
//                     fragments wave 0 leaves in LDS (double buffered), with Q and P fetched
//                     into registers a chunk ahead;
//   wave 2 ("loader") fills the ring two chunks ahead with 16-byte global->LDS loads (lane l of
//                     an instruction lands at base + 16 l, so 1 KiB of the fragment-major image
//                     per instruction, no registers).
// Ring stage s holds chunk i with i % 3 == s.  Every wave passes one barrier before the first
// chunk and one after each chunk; the loader reaches the barrier after chunk i only when
// chunk i+1 has landed, and refills the stage chunk i-1 used right after it.
template <typename E, int DK, int DV>
struct TrioSmem {
    typedef UnitLayout<E, DK, DV> U;
    static constexpr int STAGES = 3;
    static constexpr int UT_OFF = U::CHAIN_BYTES;                     // stage: [W | K^T | aux | U~ slice]
    static constexpr int STAGE_BYTES = U::CHAIN_BYTES + U::UT_SLICE_BYTES;
    static constexpr int XCH_OFF = STAGES * STAGE_BYTES;
    static constexpr int XCH_FRAGS = U::NKD + U::NKC;                 // state fragments, then U fragments
    static constexpr int BYTES = XCH_OFF + 2 * XCH_FRAGS * U::FRAG_BYTES;
    static constexpr int DMA_PER_STAGE = STAGE_BYTES / 1024;
    static_assert(DMA_PER_STAGE < 60, "outstanding-load counter");
    static_assert(BYTES <= 160 * 1024, "LDS");
};

// s_waitcnt vmcnt(N) (gfx9 encoding: vmcnt in bits 3:0 and 15:14; other counters left alone)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(((N & 0x30) << 10) | (N & 0xF) | 0x0F70);
}

template <typename E, int DK, int DV>
__global__ void __launch_bounds__(192) __attribute__((amdgpu_waves_per_eu(2, 2))) gdn_recur_trio_kernel(RecurArgs a) {
    typedef Elem<E> EL;
    typedef typename EL::Frag Frag;
    typedef UnitLayout<E, DK, DV> U;
    typedef TrioSmem<E, DK, DV> SM;
    constexpr int C = 64;
    constexpr int NS = DV / 32;
    constexpr int SPT = EL::STEPS_PER_TILE;
    constexpr int NKD = U::NKD;
    constexpr int NKC = U::NKC;
    constexpr int MT = DK / 32;

    extern __shared__ __align__(16) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lr = lane & 31;
    const int g = lane >> 5;

    const int units = a.L * a.H_v;
    const int sl = blockIdx.x % NS;
    const int chain = blockIdx.x / NS;
    const int r = a.req_order[chain / units];
    const int lh = chain % units;
    const int l = lh / a.H_v;
    const int hv = lh % a.H_v;
    const int c_begin = a.req_chunk_cu[r], c_end = a.req_chunk_cu[r + 1];
    if (c_begin == c_end) return;
    const int n_chunks = c_end - c_begin;

    const int64_t unit_stride = a.debug_same_unit ? 0 : (int64_t)units * U::UNIT_BYTES;
    const char* unit0 = a.ws_units + ((int64_t)c_begin * units + lh) * U::UNIT_BYTES;

    if (wave == 2) {
        // ------------------------------------------------------------ loader wave
        auto issue = [&](int i, int stage) {
            const int ii = i < n_chunks ? i : n_chunks - 1;   // past the end: harmless re-read
            const char* u = unit0 + ii * unit_stride;
            const char* g_chain = u + lane * 16;
            const char* g_ut = u + U::UT_OFF + sl * U::UT_SLICE_BYTES + lane * 16;
            char* dst = smem + stage * SM::STAGE_BYTES;
#pragma unroll
            for (int k = 0; k < U::CHAIN_BYTES / 1024; ++k)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g_chain + k * 1024),
                                                 (__attribute__((address_space(3))) void*)(dst + k * 1024), 16, 0, 0);
#pragma unroll
            for (int k = 0; k < U::UT_SLICE_BYTES / 1024; ++k)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g_ut + k * 1024),
                                                 (__attribute__((address_space(3))) void*)(dst + SM::UT_OFF + k * 1024), 16, 0, 0);
        };
        issue(0, 0);
        issue(1, 1);
        wait_vmcnt<SM::DMA_PER_STAGE>();        // chunk 0 has landed
        __builtin_amdgcn_s_barrier();
        int stage = 2;
        for (int i = 0; i < n_chunks; ++i) {
            issue(i + 2, stage);                // the stage chunk i-1 has just released
            stage = stage == 2 ? 0 : stage + 1;
            wait_vmcnt<SM::DMA_PER_STAGE>();    // chunk i+1 has landed
            __builtin_amdgcn_s_barrier();
        }
        wait_vmcnt<0>();
    } else if (wave == 0) {
        // ------------------------------------------------------------ chain wave
        f32x16 accS[MT];
        const int64_t head_off = ((int64_t)l * a.H_v + hv) * DV * DK + (int64_t)(32 * sl + lr) * DK;
        {
            const int slot = a.req_src_slot[r];
            if (slot >= 0) {
                const float* src = a.state_src + slot * a.src_slot_stride + head_off;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const f32x4 x = *reinterpret_cast<const f32x4*>(src + 32 * mt + 8 * b + 4 * g);
                        accS[mt][4 * b] = x[0]; accS[mt][4 * b + 1] = x[1];
                        accS[mt][4 * b + 2] = x[2]; accS[mt][4 * b + 3] = x[3];
                    }
            } else {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) accS[mt][i] = 0.f;
            }
        }
        __syncthreads();   // chunk 0 is in the ring
        int stage = 0;
        for (int i = 0; i < n_chunks; ++i) {
            const int eslot = a.chunk_emit_slot[c_begin + i];
            const char* st = smem + stage * SM::STAGE_BYTES;
            stage = stage == 2 ? 0 : stage + 1;
            const Frag* w_img = reinterpret_cast<const Frag*>(st + U::W_OFF) + lane;
            const Frag* kt_img = reinterpret_cast<const Frag*>(st + U::KT_OFF) + lane;
            const float* gamS = reinterpret_cast<const float*>(st + U::AUX_OFF);
            const float* decS = gamS + C;
            const f32x4* ut = reinterpret_cast<const f32x4*>(st + SM::UT_OFF) + lane;
            Frag* xch = reinterpret_cast<Frag*>(smem + SM::XCH_OFF) + (i & 1) * SM::XCH_FRAGS * 64 + lane;
            // [A] this chunk's W fragments and U~ accumulators: LDS reads in flight during [B]
            Frag wf[2 * NKD];
#pragma unroll
            for (int k = 0; k < 2 * NKD; ++k) wf[k] = w_img[k * 64];
            f32x16 accU[2];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const f32x4 x = ut[(rt * 4 + b) * 64];
                    accU[rt][4 * b] = x[0]; accU[rt][4 * b + 1] = x[1];
                    accU[rt][4 * b + 2] = x[2]; accU[rt][4 * b + 3] = x[3];
                }
            const float gam_last = gamS[C - 1];
            __builtin_amdgcn_sched_barrier(0);
            // [B] state -> B fragments, shared with the output wave
            Frag sf[NKD];
#pragma unroll
            for (int s = 0; s < NKD; ++s) {
                sf[s] = EL::from_acc(accS[s / SPT], s % SPT);
                xch[s * 64] = sf[s];
            }
            __builtin_amdgcn_sched_barrier(0);
            // [C] U = U~ + W S^T.  Independent accumulators alternate, so consecutive MFMAs never
            //     wait on each other; the decay of the old state (gam_C S) rides in their shadow.
#pragma unroll
            for (int s = 0; s < NKD; ++s)
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) accU[rt] = EL::mma(wf[rt * NKD + s], sf[s], accU[rt]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    accS[mt][k] *= gam_last;
                    asm volatile("" : "+v"(accS[mt][k]));   // keep the multiply here, not where its result is used
                }
#pragma unroll
            for (int k = 0; k < 2 * NKD; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, (16 * MT) / (2 * NKD), 0); // a share of the multiplies
            }
            __builtin_amdgcn_sched_barrier(0);
            // [D] K^T fragments and decay factors: in flight while U is converted
            Frag kf[MT * NKC];
#pragma unroll
            for (int k = 0; k < MT * NKC; ++k) kf[k] = kt_img[k * 64];
            f32x4 dc[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) dc[k] = *reinterpret_cast<const f32x4*>(decS + 8 * k + 4 * g);
            __builtin_amdgcn_sched_barrier(0);
            // [E] U decayed to the chunk end, as B operand of the state update
            Frag ud[NKC];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                f32x16 d = accU[rt];
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int e = 0; e < 4; ++e) d[4 * b + e] *= dc[rt * 4 + b][e];
#pragma unroll
                for (int s = 0; s < SPT; ++s) ud[rt * SPT + s] = EL::from_acc(d, s);
            }
            __builtin_amdgcn_sched_barrier(0);
            // [G] state update S^T += K^T-contraction, with [H] (plain U for the output wave)
            //     converted and written in the MFMAs' shadow
#pragma unroll
            for (int s = 0; s < NKC; ++s)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) accS[mt] = EL::mma(kf[mt * NKC + s], ud[s], accS[mt]);
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int s = 0; s < SPT; ++s) xch[(NKD + rt * SPT + s) * 64] = EL::from_acc(accU[rt], s);
            __builtin_amdgcn_sched_barrier(0);
            if (eslot >= 0) {
                float* dst = a.state_dst + eslot * a.dst_slot_stride + head_off;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const f32x4 x = {accS[mt][4 * b], accS[mt][4 * b + 1], accS[mt][4 * b + 2], accS[mt][4 * b + 3]};
                        *reinterpret_cast<f32x4*>(dst + 32 * mt + 8 * b + 4 * g) = x;
                    }
            }
            __syncthreads();   // this chunk's fragments are in LDS; its ring stage is free
        }
    } else {
        // ------------------------------------------------------------ output wave
        // Left operands of chunk i+1 are requested before chunk i's results are stored, so that
        // their memory latency is covered by a chunk of work.
        const char* unit = unit0;
        Frag qf[2 * NKD], pf[2 * NKC];
        float gm[2];
#define GDN_LOAD_QP(u_)                                                                       \
    {                                                                                         \
        const Frag* q_ = reinterpret_cast<const Frag*>((u_) + U::Q_OFF) + lane;               \
        const Frag* p_ = reinterpret_cast<const Frag*>((u_) + U::P_OFF) + lane;               \
        const float* g_ = reinterpret_cast<const float*>((u_) + U::AUX_OFF) + lr;             \
        _Pragma("unroll") for (int i_ = 0; i_ < 2 * NKD; ++i_) qf[i_] = q_[i_ * 64];          \
        _Pragma("unroll") for (int i_ = 0; i_ < SPT; ++i_) pf[i_] = p_[i_ * 64];              \
        _Pragma("unroll") for (int i_ = 0; i_ < NKC; ++i_) pf[NKC + i_] = p_[(NKC + i_) * 64]; \
        gm[0] = g_[0]; gm[1] = g_[32];                                                        \
    }
        GDN_LOAD_QP(unit)
        __syncthreads();   // matches the barrier before the first chunk
        for (int i = 0; i < n_chunks; ++i) {
            const int tok0 = a.chunk_tok0[c_begin + i];
            const int n = a.chunk_len[c_begin + i];
            const int64_t row0 = (int64_t)l * a.T_alloc + tok0;
            const char* nxt = (i + 1 < n_chunks) ? unit + unit_stride : unit;

            __syncthreads();   // the chain wave has left this chunk's state and U fragments
            const Frag* xch = reinterpret_cast<const Frag*>(smem + SM::XCH_OFF) + (i & 1) * SM::XCH_FRAGS * 64 + lane;
            Frag sf[NKD], uf[NKC];
#pragma unroll
            for (int s = 0; s < NKD; ++s) sf[s] = xch[s * 64];
#pragma unroll
            for (int s = 0; s < NKC; ++s) uf[s] = xch[(NKD + s) * 64];

            // O^T tiles of the two token tiles, their MFMA chains interleaved
            f32x16 ot[2] = {{0}, {0}};
#pragma unroll
            for (int s = 0; s < NKD; ++s)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) ot[tt] = EL::mma(sf[s], qf[tt * NKD + s], ot[tt]);
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const float sc = gm[tt] * a.scale;
#pragma unroll
                for (int k = 0; k < 16; ++k) ot[tt][k] *= sc;
            }
#pragma unroll
            for (int s = 0; s < NKC; ++s)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
                    if (s < (tt + 1) * SPT) ot[tt] = EL::mma(uf[s], pf[tt * NKC + s], ot[tt]);
            GDN_LOAD_QP(nxt)   // next chunk's operands into the registers just freed
            unit = nxt;
            store_o_t<DV>(a, row0, hv, sl, lr, g, n, ot);
        }
#undef GDN_LOAD_QP
    }
}

}  // namespace gdn
