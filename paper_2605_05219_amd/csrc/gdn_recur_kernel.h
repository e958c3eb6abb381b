// Recurrence kernel: the state-dependent part, sequential over the chunks of one chain
// (request, layer, value head).  Each wave owns a 32-column slice of d_v for the whole chain:
// the slice of the state (as S^T, d_k x 32, fp32 accumulators), of U and of O.  Rows of the
// state are independent given the chunk's W, Q, K^T and P, so waves never exchange data; a
// workgroup is NW waves (slices) of one chain sharing the staged tiles in LDS.
//
// Per chunk, with S the state at the chunk start (all products on the matrix cores, the
// state-derived operands fed from registers):
//     U  = U~ + W S^T                      [C][32]
//     O  = diag(gam) (Q S^T) + P U         [C][32]   (scale already folded into gam, P)
//     S^T <- gam_C S^T + K^T-contraction:  S^T[d_k][d_v] += sum_j K[j][d_k] dec_j U[j][d_v]
// and, when the chunk ends at a checkpoint position, S is stored to its pool slot.
#pragma once
#include "gdn_mma.h"

namespace gdn {

struct RecurArgs {
    const void* q;
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

template <typename E, int DK, int DV, int NW>
__global__ void __launch_bounds__(64 * NW) gdn_recur_kernel(RecurArgs a) {
    typedef Elem<E> EL;
    typedef typename EL::In In;
    typedef typename EL::Frag Frag;
    typedef UnitLayout<E, DK, DV> U;
    constexpr int C = 64;
    constexpr int NT = 64 * NW;
    constexpr int NS = DV / 32;              // slices per chain
    constexpr int SG = NS / NW;              // workgroups per chain
    constexpr int SPT = EL::STEPS_PER_TILE;
    constexpr int NKD = DK / EL::KSTEP;      // steps over d_k
    constexpr int MT = DK / 32;              // state tiles per slice
    constexpr int Q_LD = DK + EL::PAD;
    static_assert(NS % NW == 0, "slices must split evenly over workgroups");

    extern __shared__ __align__(16) char smem[];
    const E* Wt = reinterpret_cast<const E*>(smem + U::W_OFF);
    const E* KTs = reinterpret_cast<const E*>(smem + U::KT_OFF);
    const E* Pt = reinterpret_cast<const E*>(smem + U::P_OFF);
    const float* gamS = reinterpret_cast<const float*>(smem + U::AUX_OFF);
    const float* decS = gamS + C;
    E* Qs = reinterpret_cast<E*>(smem + U::STAGED_BYTES);

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
    const int hq = hv / (a.H_v / a.H_qk);
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

    for (int c = c_begin; c < c_end; ++c) {
        const int tok0 = a.chunk_tok0[c];
        const int n = a.chunk_len[c];
        const int64_t row0 = (int64_t)l * a.T_alloc + tok0;
        const char* unit = a.ws_units + ((int64_t)(c * a.L + l) * a.H_v + hv) * U::UNIT_BYTES;

        __syncthreads();  // the previous chunk's tiles are no longer read
        {
            const uint4* src = reinterpret_cast<const uint4*>(unit);
            uint4* dst = reinterpret_cast<uint4*>(smem);
            for (int i = tid; i < U::STAGED_BYTES / 16; i += NT) dst[i] = src[i];
            const In* qg = reinterpret_cast<const In*>(a.q);
            constexpr int VPR = DK / 8;
            for (int u = tid; u < C * VPR; u += NT) {
                const int i = u / VPR, d0 = (u % VPR) * 8;
                float qv[8];
                if (i < n) {
                    EL::load8(qg + ((row0 + i) * a.H_qk + hq) * DK + d0, qv);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) qv[e] = 0.f;
                }
                EL::store4(Qs + i * Q_LD + d0, qv[0], qv[1], qv[2], qv[3]);
                EL::store4(Qs + i * Q_LD + d0 + 4, qv[4], qv[5], qv[6], qv[7]);
            }
        }
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
        __syncthreads();

        // state as the B operand of the two products that contract over d_k
        Frag sf[NKD];
#pragma unroll
        for (int s = 0; s < NKD; ++s) sf[s] = EL::from_acc(accS[s / SPT], s % SPT);

        f32x16 accO[2];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const E* wr = Wt + (32 * rt + lr) * U::W_LD;
            const E* qr = Qs + (32 * rt + lr) * Q_LD;
            f32x16 o = {0};
#pragma unroll
            for (int s = 0; s < NKD; ++s) {
                accU[rt] = EL::mma(EL::load(wr, s, g), sf[s], accU[rt]);
                o = EL::mma(EL::load(qr, s, g), sf[s], o);
            }
            // rows of Q S^T scale with gam_i (and the output scale)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const f32x4 gm = *reinterpret_cast<const f32x4*>(gamS + 32 * rt + 8 * b + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) o[4 * b + e] *= gm[e] * a.scale;
            }
            accO[rt] = o;
        }

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

        // O += P U (P is lower triangular: token tile 0 only sees key tile 0), then store
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const E* pr = Pt + (32 * rt + lr) * U::P_LD;
#pragma unroll
            for (int s = 0; s < (rt + 1) * SPT; ++s) accO[rt] = EL::mma(EL::load(pr, s, g), uf[s], accO[rt]);
            const int col = 32 * sl + lr;
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                const int row = 32 * rt + acc_row(idx, g);
                if (row < n) {
                    const int64_t off = ((row0 + row) * a.H_v + hv) * DV + col;
                    if (a.o_bf16) reinterpret_cast<uint16_t*>(a.o)[off] = f32_to_bf16_rne(accO[rt][idx]);
                    else reinterpret_cast<float*>(a.o)[off] = accO[rt][idx];
                }
            }
        }

        // state update: S^T = gam_C S^T + sum_j K^T[.][j] (dec_j U[j][.])
        const float gam_last = gamS[C - 1];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int i = 0; i < 16; ++i) accS[mt][i] *= gam_last;
            const E* kr = KTs + (32 * mt + lr) * U::KT_LD;
#pragma unroll
            for (int s = 0; s < 2 * SPT; ++s) accS[mt] = EL::mma(EL::load(kr, s, g), ud[s], accS[mt]);
        }

        // checkpoint emission: exact state after the last token of this chunk
        const int eslot = a.chunk_emit_slot[c];
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
    }
}

template <typename E, int DK, int DV>
constexpr int recur_smem_bytes() {
    return UnitLayout<E, DK, DV>::STAGED_BYTES + 64 * (DK + Elem<E>::PAD) * (int)sizeof(E);
}

}  // namespace gdn
