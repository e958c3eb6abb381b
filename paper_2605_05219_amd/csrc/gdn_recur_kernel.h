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
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// STAGED: the workgroup copies the unit's fragment image to LDS once per chunk and its NW
// waves (d_v slices) read fragments from there, the next image being prefetched into registers
// meanwhile.  !STAGED (one wave per workgroup, nothing to share): fragments are loaded from
// global memory straight into registers, no LDS, no barriers.
template <typename E, int DK, int DV, int NW, bool STAGED>
__global__ void __launch_bounds__(64 * NW) gdn_recur_kernel(RecurArgs a) {
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
    static_assert(STAGED || NW == 1, "the direct variant runs one wave per workgroup");

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
        if (STAGED) {
            __syncthreads();  // the previous chunk's image is no longer read
            u32x4* dst = reinterpret_cast<u32x4*>(smem) + tid;
#pragma unroll
            for (int i = 0; i < NFULL; ++i) dst[i * NT] = pre[i];
            if (TAIL > 0 && tid < TAIL) dst[NFULL * NT] = pre_tail;
            __syncthreads();
            // (the last chunk re-reads its own image: no branch around the register loads)
            GDN_PREFETCH_IMAGE((c + 1 < c_end) ? unit + unit_stride : unit)
            img = smem;
        } else {
            img = unit;
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

        // O = diag(gam) (Q S^T) + P U with the state of the chunk start (sf), off the chain
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            f32x16 o = {0};
#pragma unroll
            for (int s = 0; s < NKD; ++s) o = EL::mma(q_img[(rt * NKD + s) * 64], sf[s], o);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const f32x4 gm = *reinterpret_cast<const f32x4*>(gamS + 32 * rt + 8 * b + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) o[4 * b + e] *= gm[e] * a.scale;
            }
            // P is lower triangular: token tile 0 only sees key tile 0
#pragma unroll
            for (int s = 0; s < (rt + 1) * SPT; ++s) o = EL::mma(p_img[(rt * NKC + s) * 64], uf[s], o);
            const int col = 32 * sl + lr;
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                const int row = 32 * rt + acc_row(idx, g);
                if (row < n) {
                    const int64_t off = ((row0 + row) * a.H_v + hv) * DV + col;
                    if (a.o_bf16) reinterpret_cast<uint16_t*>(a.o)[off] = f32_to_bf16_rne(o[idx]);
                    else reinterpret_cast<float*>(a.o)[off] = o[idx];
                }
            }
        }
    }
}

#undef GDN_PREFETCH_IMAGE

template <typename E, int DK, int DV>
constexpr int recur_smem_bytes(bool staged) {
    return staged ? UnitLayout<E, DK, DV>::STAGED_BYTES : 0;
}

}  // namespace gdn
