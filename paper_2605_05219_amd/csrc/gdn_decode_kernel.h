// Single-token update of the recurrent states in their pool slots (decode step): for every
// (request, layer, value head), with S the d_v x d_k fp32 state, one token (q, k, v, a, b):
//     S~ = a S;   u = b (v - S~ k);   S = S~ + u k^T;   o = scale * S q
// The rows of S are independent: row i needs the two dot products S_i.k and S_i.q of the OLD
// row, from which  u_i = b (v_i - a S_i.k),  S_i <- a S_i + u_i k,  o_i = scale (a S_i.q + u_i k.q).
// So each row is read once and written once: the kernel is bound by HBM traffic (2 x state
// bytes).  A row is spread over d_k / 4 lanes (16-byte accesses, a wave covers 1 KiB of
// consecutive memory per pass); the dot products are reduced across those lanes with xor
// shuffles, several rows in flight per lane to cover their latency.  NT: the state rows are read and written with
// non-temporal accesses, which is what a call wants whose states exceed the memory-side cache (1024 states of 1 MiB:
// 6.1 against 5.6 TB/s), and not one whose states fit it and are touched again by the next step (256 states: 6.3 against
// 6.8 TB/s); the host decides by the bytes a call touches.
#pragma once
#include "gdn_mma.h"


namespace gdn {

struct DecodeArgs {
    const void* q;
    const void* k;
    const void* v;
    const void* beta;
    const void* gate;
    float* pool;
    void* o;
    int64_t slot_stride;     // floats
    int64_t T_alloc;         // token rows per layer in q, k, v, beta, gate, o
    int32_t req_base;        // first request of this launch
    int32_t L, H_qk, H_v;
    float scale;
    int32_t o_bf16;
};

constexpr int DECODE_IDS = 256;
struct DecodeIds {
    int32_t slot[DECODE_IDS];
};

template <typename E, int DK, int DV, bool NT>
__global__ void __launch_bounds__(256) gdn_decode_kernel(DecodeArgs a, DecodeIds ids) {
    typedef Elem<E> EL;
    typedef typename EL::In In;
    constexpr int LPR = DK / 4;              // lanes per row
    constexpr int RPP = 64 / LPR;            // rows per wave pass
    constexpr int ROWS_PER_WAVE = 8;
    constexpr int NP = ROWS_PER_WAVE / RPP;  // passes, all in flight together
    static_assert(DV % 32 == 0 && ROWS_PER_WAVE % RPP == 0, "row blocking");

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane % LPR, rr = lane / LPR;
    const int lh = blockIdx.y;
    const int l = lh / a.H_v, hv = lh % a.H_v;
    const int hq = hv / (a.H_v / a.H_qk);
    const int req = a.req_base + blockIdx.z;
    const int64_t tok = (int64_t)l * a.T_alloc + req;

    const In* kp = reinterpret_cast<const In*>(a.k) + (tok * a.H_qk + hq) * DK + 4 * c;
    const In* qp = reinterpret_cast<const In*>(a.q) + (tok * a.H_qk + hq) * DK + 4 * c;
    float k4[4], q4[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) { k4[e] = EL::widen(kp[e]); q4[e] = EL::widen(qp[e]); }
    const float av = EL::widen(reinterpret_cast<const In*>(a.gate)[tok * a.H_v + hv]);
    const float bv = EL::widen(reinterpret_cast<const In*>(a.beta)[tok * a.H_v + hv]);

    const int row0 = 32 * blockIdx.x + ROWS_PER_WAVE * wave + rr;
    float* S = a.pool + (int64_t)ids.slot[blockIdx.z] * a.slot_stride + ((int64_t)l * a.H_v + hv) * DV * DK;
    const In* vp = reinterpret_cast<const In*>(a.v) + (tok * a.H_v + hv) * DV;

    f32x4 s[NP];
    float vr[NP], pk[NP], pq[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int row = row0 + p * RPP;
        s[p] = NT ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(S + (int64_t)row * DK + 4 * c)) : *reinterpret_cast<const f32x4*>(S + (int64_t)row * DK + 4 * c);
        vr[p] = EL::widen(vp[row]);
    }
    float kq = k4[0] * q4[0] + k4[1] * q4[1] + k4[2] * q4[2] + k4[3] * q4[3];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        pk[p] = s[p][0] * k4[0] + s[p][1] * k4[1] + s[p][2] * k4[2] + s[p][3] * k4[3];
        pq[p] = s[p][0] * q4[0] + s[p][1] * q4[1] + s[p][2] * q4[2] + s[p][3] * q4[3];
    }
#pragma unroll
    for (int d = 1; d < LPR; d <<= 1) {
        kq += __shfl_xor(kq, d, 64);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            pk[p] += __shfl_xor(pk[p], d, 64);
            pq[p] += __shfl_xor(pq[p], d, 64);
        }
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int row = row0 + p * RPP;
        const float u = bv * (vr[p] - av * pk[p]);
        f32x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = av * s[p][e] + u * k4[e];
        if (NT) __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(S + (int64_t)row * DK + 4 * c)); else *reinterpret_cast<f32x4*>(S + (int64_t)row * DK + 4 * c) = t;
        if (c == 0) {
            const float ov = a.scale * (av * pq[p] + u * kq);
            const int64_t oi = (tok * a.H_v + hv) * DV + row;
            if (a.o_bf16) {
                uint32_t x = __float_as_uint(ov);
                uint16_t h;
                if ((x & 0x7fffffffu) > 0x7f800000u) h = (uint16_t)((x >> 16) | 0x40);
                else h = (uint16_t)((x + 0x7fffu + ((x >> 16) & 1u)) >> 16);
                reinterpret_cast<uint16_t*>(a.o)[oi] = h;
            } else {
                reinterpret_cast<float*>(a.o)[oi] = ov;
            }
        }
    }
}

}  // namespace gdn
