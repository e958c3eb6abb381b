// Chunk preparation kernel: everything of a 64-token chunk that does not depend on the
// recurrent state.  A workgroup (4 waves) handles one (chunk, layer, value head) at a time; a
// launch covers one slab, i.e. up to R consecutive chunks of every request, with as many
// workgroups as the chip holds at once, each looping over its share of the slab.
//
// With g_i the running sum of log a inside the chunk, gam_i = exp(g_i), and the chunk-local
// form of the gated delta rule
//     S_i = gam_i S_0 + sum_{j<=i} exp(g_i-g_j) u_j k_j^T ,   (I + L) U = diag(b)(V - diag(gam) K S_0^T)
//     L_ij = b_i exp(g_i-g_j) (k_i.k_j)  for j < i,
// it produces, with T = (I+L)^-1 (fp32):
//     W  = -T diag(b gam) K          [C][d_k]   (so that U = U~ + W S_0^T)
//     U~ =  T diag(b) V              [C][d_v]   in the recurrence kernel's accumulator order (fp16 for
//                                               16-bit inputs, fp32 for fp32 inputs)
//     P_ij = scale * exp(g_i-g_j) (q_i.k_j), j <= i   [C][C]
//     Q, K^T diag(dec) with dec_i = exp(g_C - g_i) (the decay to the chunk end rides on K, so
//     the recurrence uses one conversion of U for both of its uses), gam_i, bookkeeping words
// W, Q, K^T and P leave in fragment-major order (see UnitLayout).  A product's accumulator tile
// already holds, lane for lane, the fragments of its transpose, so W and P go from the
// accumulators to global memory with coalesced stores; Q and K^T fragments are the operands
// this kernel loaded for its own products.
// Tokens past the chunk's valid length are identity tokens (a = 1, b = 0, k = q = v = 0), which
// leave the state untouched, so a short chunk needs no special arithmetic.
#pragma once
#include "gdn_mma.h"

namespace gdn {

struct PrepArgs {
    const void* q;
    const void* k;
    const void* v;
    const void* beta;
    const void* gate;
    const int32_t* chunk_tok0;
    const int32_t* chunk_len;
    const int32_t* chunk_emit_slot;
    const int32_t* req_chunk_cu;
    char* ws_units;       // this slab's units: (request r, round j, l, h) at (((r * R + j) * L + l) * H_v + h) * UNIT_BYTES
    int32_t slab_begin;   // first chunk round of the slab (rounds are counted per request)
    int32_t R;            // chunk rounds per slab
    int32_t n_req;
    int32_t L, H_qk, H_v;
    int64_t T_alloc;
    float scale;
    // Host tier (first launch of a call only, else n_copy_wgs = 0): the last n_copy_wgs workgroups
    // of the grid copy the start states from device-accessible pinned host memory to the staging
    // area, so the transfer rides under this launch.
    const float* host_pool;          // device-side address of the pinned host pool
    int64_t host_slot_stride;        // floats
    const int32_t* staged_slot;      // [n_staged] host slot of the i-th staged state
    float* staging;                  // [n_staged][slot_elems]
    int64_t slot_elems;
    int32_t n_staged;
    int32_t n_copy_wgs;
};

// D(16x16) += A(16x16) * B(16x16), fp32 MFMA 16x16x4.  Lane (m = l & 15, g4 = l >> 4).
// A and B are blocks of the fp32 matrix Lf (leading dimension LD) in LDS.
template <int LD>
__device__ __forceinline__ f32x4 mm16_ll(f32x4 acc, const float* A, const float* B, int m, int g4) {
#pragma unroll
    for (int s = 0; s < 4; ++s)
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(A[m * LD + 4 * s + g4], B[(4 * s + g4) * LD + m], acc, 0, 0, 0);
    return acc;
}
// Same with B taken from an accumulator tile (rows 4*g4+e are the contraction index).
template <int LD>
__device__ __forceinline__ f32x4 mm16_lr(f32x4 acc, const float* A, const f32x4 B, int m, int g4) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(A[m * LD + 4 * g4 + e], B[e], acc, 0, 0, 0);
    return acc;
}

// Same with both operands in registers: D += A B given the accumulator-layout tiles of A^T and of B
// (lane (m, g4) holds rows 4 g4 .. 4 g4 + 3 of column m; step e contracts over the indices 4 g4' + e).
__device__ __forceinline__ f32x4 mm16_rr(f32x4 acc, const f32x4 At, const f32x4 B) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(At[e], B[e], acc, 0, 0, 0);
    return acc;
}

// (I + D)^-1 for a strictly lower triangular 16x16 block D of an fp32 matrix in LDS, by the nilpotent
// product (I + D^8)(I + D^4)(I + D^2)(I - D) (exact: D^16 = 0), entirely in registers: every power is
// carried as the accumulator tiles of itself and of its transpose, which is what a product needs of its
// left and right operand, so nothing goes back through LDS (eight 16x16 products on v_mfma_f32_16x16x4_f32).
// Returns the accumulator tile of the inverse: element e of lane (m, g4) is entry (4 g4 + e, m).
template <int LD>
__device__ __forceinline__ f32x4 inv16_unit_lower(const float* D, int m, int g4) {
    f32x4 d, y;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        d[e] = D[(4 * g4 + e) * LD + m];
        y[e] = ((4 * g4 + e) == m ? 1.f : 0.f) - d[e];
    }
    const f32x4 dt = *reinterpret_cast<const f32x4*>(D + m * LD + 4 * g4);   // tile of D^T: row m of D
    const f32x4 zero = {0, 0, 0, 0};
    const f32x4 p2 = mm16_rr(zero, dt, d), p2t = mm16_rr(zero, d, dt);       // D^2 and its transpose
    y = mm16_rr(y, p2t, y);                                                  // (I + D^2)(I - D)
    const f32x4 p4 = mm16_rr(zero, p2t, p2), p4t = mm16_rr(zero, p2, p2t);
    y = mm16_rr(y, p4t, y);
    const f32x4 p8t = mm16_rr(zero, p4, p4t);
    return mm16_rr(y, p8t, y);
}

template <typename E, int DK, int DV>
struct PrepSmem {
    typedef UnitLayout<E, DK, DV> U;
    static constexpr int C = 64;
    static constexpr int PAD = Elem<E>::PAD;
    static constexpr int LF_LD = C + 4;   // rows 16-byte aligned
    static constexpr int a16(int x) { return (x + 15) / 16 * 16; }
    static constexpr int KT_LD = C + PAD;
    static constexpr int VT_LD = C + PAD;
    static constexpr int cmax(int x, int y) { return x > y ? x : y; }
    // region A: K [C][DK+PAD]; once the first products are done, V^T [DV][C+PAD]
    static constexpr int A_OFF = 0;
    static constexpr int A_BYTES = cmax(a16(C * (DK + PAD) * (int)sizeof(E)), a16(DV * VT_LD * (int)sizeof(E)));
    static constexpr int B_OFF = A_OFF + A_BYTES;
    // region B: Q [C][DK+PAD]
    static constexpr int B_BYTES = a16(C * (DK + PAD) * (int)sizeof(E));
    static constexpr int KT_OFF = B_OFF + B_BYTES;
    static constexpr int KT_BYTES = a16(DK * KT_LD * (int)sizeof(E));
    static constexpr int LF_OFF = KT_OFF + KT_BYTES;
    static constexpr int LF_BYTES = a16(C * LF_LD * (int)sizeof(float));
    static constexpr int SM_OFF = LF_OFF + LF_BYTES;  // g[C], b[C], gam[C], dec[C], -b gam [C]
    static constexpr int BYTES = SM_OFF + 5 * C * (int)sizeof(float);
};

// The work of one preparation workgroup: workgroup `wg` of `n_prep_wgs` that share a launch's items.
template <typename E, int DK, int DV>
__device__ __forceinline__ void prep_body(const PrepArgs& a, const int wg, const int n_prep_wgs) {
    typedef Elem<E> EL;
    typedef typename EL::In In;
    typedef typename EL::Frag Frag;
    typedef UnitLayout<E, DK, DV> U;
    typedef PrepSmem<E, DK, DV> SM;
    constexpr int C = 64;
    constexpr int PAD = EL::PAD;
    constexpr int K_LD = DK + PAD;
    constexpr int KT_LD = SM::KT_LD;
    constexpr int VT_LD = SM::VT_LD;
    constexpr int LF_LD = SM::LF_LD;

    extern __shared__ __align__(16) char smem[];
    E* Ks = reinterpret_cast<E*>(smem + SM::A_OFF);
    E* Qs = reinterpret_cast<E*>(smem + SM::B_OFF);
    E* KTs = reinterpret_cast<E*>(smem + SM::KT_OFF);
    E* VTs = reinterpret_cast<E*>(smem + SM::A_OFF);       // after the first products
    float* Lf = reinterpret_cast<float*>(smem + SM::LF_OFF);
    float* gS = reinterpret_cast<float*>(smem + SM::SM_OFF);
    float* bS = gS + C;
    float* gamS = bS + C;
    float* decS = gamS + C;
    float* bgS = decS + C;   // -b gam

    const int tid = threadIdx.x;
    const int lane_ = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: say so
    const int lr_ = lane_ & 31;
    const int g_ = lane_ >> 5;
    constexpr int SPT = EL::STEPS_PER_TILE;
    const In* const qg = reinterpret_cast<const In*>(a.q);
    const In* const kg = reinterpret_cast<const In*>(a.k);
    const In* const vg = reinterpret_cast<const In*>(a.v);

    // Work items of the launch: u = x * units + lh with x = r * R + j (chunk round slab_begin + j
    // of request r, skipped if the request has no such round).  The workgroup takes items
    // wg, wg + n_prep_wgs, ... and fetches the inputs of its next item while it
    // works on the current one.
    const int units = a.L * a.H_v;
    const int total = a.n_req * a.R * units;
    struct Item { int u, c, lh, x, tok0, n; };
    auto locate = [&](int u) -> Item {
        Item it;
        it.c = -1; it.lh = 0; it.x = 0; it.tok0 = 0; it.n = 0;
        for (;; u += n_prep_wgs) {
            it.u = u;
            if (u >= total) return it;
            it.x = u / units;
            it.lh = u - it.x * units;
            const int r = it.x / a.R;
            it.c = a.req_chunk_cu[r] + a.slab_begin + (it.x - r * a.R);
            if (it.c < a.req_chunk_cu[r + 1]) break;
        }
        it.tok0 = a.chunk_tok0[it.c];
        it.n = a.chunk_len[it.c];
        return it;
    };
    // A thread owns 4-token x 8-column blocks of K, Q and V.
    constexpr int KB = (C / 4) * (DK / 8), VB = (C / 4) * (DV / 8);   // blocks of K (and Q), of V
    static_assert(KB <= 256 && VB <= 256, "one block per thread at most");
    const int tg_ = tid / (DK / 8), d0_ = (tid % (DK / 8)) * 8;
    const int tgv_ = tid / (DV / 8), d0v_ = (tid % (DV / 8)) * 8;
    typedef typename EL::Raw8 Raw8;
    // (16-bit inputs only: the fp32 fetch registers would not fit next to the working set)
    constexpr bool PREFETCH = sizeof(In) == 2;
    Raw8 kraw[4], qraw[4], vraw[4];
    In graw = In(), braw = In();
    auto fetch_kq = [&](const Item& it) {
        const int l = it.lh / a.H_v, hq = (it.lh % a.H_v) / (a.H_v / a.H_qk);
        const int64_t row0 = (int64_t)l * a.T_alloc + it.tok0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = 4 * tg_ + r;
            if (tid < KB && i < it.n) {
                const int64_t off = ((row0 + i) * a.H_qk + hq) * DK + d0_;
                kraw[r] = EL::load_raw(kg + off);
                qraw[r] = EL::load_raw(qg + off);
            } else {
                kraw[r] = EL::zero_raw();
                qraw[r] = EL::zero_raw();
            }
        }
    };
    auto fetch_v = [&](const Item& it) {
        const int l = it.lh / a.H_v, hv = it.lh % a.H_v;
        const int64_t row0 = (int64_t)l * a.T_alloc + it.tok0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int iv = 4 * tgv_ + r;
            if (tid < VB && iv < it.n) vraw[r] = EL::load_raw(vg + ((row0 + iv) * a.H_v + hv) * DV + d0v_);
            else vraw[r] = EL::zero_raw();
        }
        if (wave == 0 && lane_ < it.n) {
            const int64_t gi = (row0 + lane_) * a.H_v + hv;
            graw = reinterpret_cast<const In*>(a.gate)[gi];
            braw = reinterpret_cast<const In*>(a.beta)[gi];
        }
    };

    Item cur = locate(wg);
    if (cur.u >= total) return;
    // The fp32 triangular matrix: its upper right 32x32 tile is never written and must read as 0
    // (every other entry on or above the diagonal is rewritten with an exact 0 for each item).
    for (int i = tid; i < C * LF_LD; i += 256) Lf[i] = 0.f;
    fetch_kq(cur);
    fetch_v(cur);
    Item nxt = locate(cur.u + n_prep_wgs);

  for (;;) {
    // The thread's coordinates are made opaque once per item: otherwise every address of the
    // unrolled tile accesses below is hoisted out of this loop and held in a register of its
    // own for the whole kernel.
    int tid_p = tid, lane = lane_, lr = lr_, g = g_, tg = tg_, d0 = d0_, tgv = tgv_, d0v = d0v_;
    pin(tid_p); pin(lane); pin(lr); pin(g); pin(tg); pin(d0); pin(tgv); pin(d0v);
    const int c = cur.c;
    const int lh = cur.lh;
    const int tok0 = cur.tok0;
    const int n = cur.n;
    char* unit = a.ws_units + ((int64_t)cur.x * units + lh) * U::UNIT_BYTES;
    Frag* w_img = reinterpret_cast<Frag*>(unit + U::W_OFF);
    Frag* q_img = reinterpret_cast<Frag*>(unit + U::Q_OFF);
    Frag* kt_img = reinterpret_cast<Frag*>(unit + U::KT_OFF);
    Frag* p_img = reinterpret_cast<Frag*>(unit + U::P_OFF);

    // ---- gates: g_i = inclusive running sum of log a (wave 0), b_i; identity beyond n
    if (wave == 0) {
        float la = 0.f, b = 0.f;
        if (lane < n) {
            la = fmaxf(EL::log_(EL::widen(graw)), -88.f);
            b = EL::widen(braw);
        }
        const float s = wave_running_sum(la);
        const float g_last = wave_last_lane(s);
        gS[lane] = s;
        bS[lane] = b;
        const float gam = EL::exp_(s);
        gamS[lane] = gam;
        decS[lane] = EL::exp_(g_last - s);
        bgS[lane] = -b * gam;
    }

    // ---- stage K, Q (row-major) and K^T (token-contiguous), converted to E; the transposed
    //      copy goes out as 4-token runs.  V stays in registers; its transposed tile takes K's
    //      place once K is dead.
    if (tid_p < KB) {
        float kv[4][8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = 4 * tg + r;
            float qv[8];
            EL::unpack(kraw[r], kv[r]);
            EL::unpack(qraw[r], qv);
            EL::store4(Ks + i * K_LD + EL::slot4(d0), kv[r][0], kv[r][1], kv[r][2], kv[r][3]);
            EL::store4(Ks + i * K_LD + EL::slot4(d0 + 4), kv[r][4], kv[r][5], kv[r][6], kv[r][7]);
            EL::store4(Qs + i * K_LD + EL::slot4(d0), qv[0], qv[1], qv[2], qv[3]);
            EL::store4(Qs + i * K_LD + EL::slot4(d0 + 4), qv[4], qv[5], qv[6], qv[7]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e)
            EL::store4(KTs + (d0 + e) * KT_LD + EL::slot4(4 * tg), kv[0][e], kv[1][e], kv[2][e], kv[3][e]);
    }
    if (PREFETCH && nxt.u < total) fetch_kq(nxt);   // K and Q of the next item travel during the rest of this one
    __syncthreads();

    // ---- K K^T -> L (fp32) and K Q^T -> P fragments
    //      wave 0: KK(0,0) KQ(0,0)   wave 1: KK(1,0)   wave 2: KK(1,1) KQ(1,1)   wave 3: KQ(0,1)
    constexpr int NKD = DK / EL::KSTEP;
    {
        int kk_mi = -1, kk_nj = -1, p_mj = -1, p_ni = -1;
        if (wave == 0) { kk_mi = 0; kk_nj = 0; p_mj = 0; p_ni = 0; }
        if (wave == 1) { kk_mi = 1; kk_nj = 0; }
        if (wave == 2) { kk_mi = 1; kk_nj = 1; p_mj = 1; p_ni = 1; }
        if (wave == 3) { p_mj = 0; p_ni = 1; }
        if (kk_mi >= 0) {
            f32x16 acc = {0};
            const E* ar = Ks + (32 * kk_mi + lr) * K_LD;
            const E* br = Ks + (32 * kk_nj + lr) * K_LD;
#pragma unroll
            for (int s = 0; s < NKD; ++s) acc = EL::mma(EL::load(ar, s, g), EL::load(br, s, g), acc);
            const int j = 32 * kk_nj + lr;
            const float gj = gS[j];
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                const int i = 32 * kk_mi + acc_row(idx, g);
                const float val = bS[i] * EL::exp_(fminf(gS[i] - gj, 0.f)) * acc[idx];
                Lf[i * LF_LD + j] = (j < i) ? val : 0.f;
            }
        }
        if (p_mj >= 0) {
            // D[key j][query i]: the accumulators of lane (i, g) are row i of P at the key
            // positions that lane carries as an A operand, i.e. P's fragments (row tile p_ni).
            f32x16 acc = {0};
            const E* ar = Ks + (32 * p_mj + lr) * K_LD;   // rows: key token j
            const E* br = Qs + (32 * p_ni + lr) * K_LD;   // rows: query token i
            const bool write_q = (p_mj == p_ni);          // waves 0 and 2 also emit Q's fragments
#pragma unroll
            for (int s = 0; s < NKD; ++s) {
                const Frag qf = EL::load(br, s, g);
                if (write_q) q_img[(p_ni * NKD + s) * 64 + lane] = qf;
                acc = EL::mma(EL::load(ar, s, g), qf, acc);
            }
            const int i = 32 * p_ni + lr;
            const float gi = gS[i];
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                const int j = 32 * p_mj + acc_row(idx, g);
                const float val = a.scale * EL::exp_(fminf(gi - gS[j], 0.f)) * acc[idx];
                acc[idx] = (j <= i) ? val : 0.f;
            }
#pragma unroll
            for (int sub = 0; sub < SPT; ++sub)
                p_img[(p_ni * U::NKC + p_mj * SPT + sub) * 64 + lane] = EL::from_acc(acc, sub);
        }
    }
    __syncthreads();  // L is complete; K, Q in LDS are dead

    // ---- V^T into K's place (read by the last product, several barriers from here)
    if (tid_p < VB) {
        float vv[4][8];
#pragma unroll
        for (int r = 0; r < 4; ++r) EL::unpack(vraw[r], vv[r]);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            EL::store4(VTs + (d0v + e) * VT_LD + EL::slot4(4 * tgv), vv[0][e], vv[1][e], vv[2][e], vv[3][e]);
    }
    if (PREFETCH && nxt.u < total) fetch_v(nxt);    // V and the gates of the next item

    // ---- T = (I + L)^-1, fp32, by 16x16 blocks.  Stage 1: the four diagonal blocks, one per
    //      wave.  A strictly lower triangular 16x16 block D has D^16 = 0, so
    //          (I + D)^-1 = (I + D^8)(I + D^4)(I + D^2)(I - D)
    //      exactly: squarings and products on the matrix cores instead of a sixteen-step
    //      substitution, all in registers (see inv16_unit_lower).
    const int m16 = lane & 15, g4 = lane >> 4;
    {
        float* const D = Lf + (16 * wave) * LF_LD + 16 * wave;
        const f32x4 y = inv16_unit_lower<LF_LD>(D, m16, g4);
#pragma unroll
        for (int e = 0; e < 4; ++e) D[(4 * g4 + e) * LF_LD + m16] = y[e];
    }
    __syncthreads();  // diagonal blocks of T in place

    auto blk = [&](int br, int bc) -> const float* { return Lf + (16 * br) * LF_LD + 16 * bc; };
    // Stage 2: T_10 = -T_11 (L_10 T_00) on wave 0, T_32 = -T_33 (L_32 T_22) on wave 1.
    if (wave < 2) {
        const int ra = 2 * wave + 1, rb = 2 * wave;
        f32x4 m = {0, 0, 0, 0};
        m = mm16_ll<LF_LD>(m, blk(ra, rb), blk(rb, rb), m16, g4);
        f32x4 r = {0, 0, 0, 0};
        r = mm16_lr<LF_LD>(r, blk(ra, ra), m, m16, g4);
#pragma unroll
        for (int e = 0; e < 4; ++e) Lf[(16 * ra + 4 * g4 + e) * LF_LD + 16 * rb + m16] = -r[e];
    }
    __syncthreads();
    // Stage 3: the 32x32 block below the diagonal.  Wave w owns T_ab, a = 2 + w/2, b = w%2:
    //   X_cb = L_c0 T_0b + L_c1 T_1b (c = 2, 3);  T_2b = -T_22 X_2b;  T_3b = -(T_32 X_2b + T_33 X_3b).
    {
        const int ra = 2 + (wave >> 1), rb = wave & 1;
        f32x4 x2 = {0, 0, 0, 0};
        if (rb == 0) x2 = mm16_ll<LF_LD>(x2, blk(2, 0), blk(0, 0), m16, g4);
        x2 = mm16_ll<LF_LD>(x2, blk(2, 1), blk(1, rb), m16, g4);
        f32x4 r = {0, 0, 0, 0};
        r = mm16_lr<LF_LD>(r, blk(ra, 2), x2, m16, g4);
        if (ra == 3) {
            f32x4 x3 = {0, 0, 0, 0};
            if (rb == 0) x3 = mm16_ll<LF_LD>(x3, blk(3, 0), blk(0, 0), m16, g4);
            x3 = mm16_ll<LF_LD>(x3, blk(3, 1), blk(1, rb), m16, g4);
            r = mm16_lr<LF_LD>(r, blk(3, 3), x3, m16, g4);
        }
        // The 32x32 block below the diagonal tiles is stored in the tile ABOVE them (rows 0..31, columns 32..63),
        // which nothing else uses: no L block that another wave still reads is overwritten, so no barrier.
#pragma unroll
        for (int e = 0; e < 4; ++e) Lf[(16 * (ra - 2) + 4 * g4 + e) * LF_LD + 32 + 16 * rb + m16] = -r[e];
    }
    __syncthreads();  // T complete in Lf

    // T stays in fp32: the operand fragments of Tb = T diag(b) and Tbg = -T diag(b gam) are made
    // from its rows on use (the scale, the conversion), so no converted copy is written and no
    // barrier separates T from its two uses.  Entries above the diagonal inside the tiles that
    // are read are exact zeros (written so by the K K^T epilogue and kept by the inversion); the
    // tile above the diagonal tiles holds the block below them.
    // ---- W^T tile (mt, nt): D[d_k][token i] = sum_j K^T[d_k][j] Tbg[i][j].  The accumulators of
    //      lane (i, g) are W's fragments of row tile nt, steps SPT*mt ..; the A operands are
    //      K^T's fragments.  T is lower triangular: token tile 0 only contracts over j < 32.
    constexpr int NKC = C / EL::KSTEP;
    for (int t = wave; t < (DK / 32) * 2; t += 4) {
        const int mt = t % (DK / 32), nt = t / (DK / 32);   // a wave's tiles: one of each token tile where possible
        f32x16 acc = {0};
        const E* ar = KTs + (32 * mt + lr) * KT_LD;
        const float* br = Lf + (32 * nt + lr) * LF_LD;
        const float* br10 = Lf + lr * LF_LD + 32;   // rows 32.., columns 0..31 of T live above the diagonal tiles
        const int ns = (nt == 0) ? NKC / 2 : NKC;
#pragma unroll
        for (int s = 0; s < NKC; ++s)
            if (s < ns) {
                const Frag kf = EL::load(ar, s, g);
                if (nt == 1) kt_img[(mt * NKC + s) * 64 + lane] = EL::scale(kf, decS, s, g);   // decayed to the chunk end
                acc = EL::mma(kf, EL::load_scaled((nt == 1 && s < NKC / 2) ? br10 : br, bgS, s, g), acc);
            }
#pragma unroll
        for (int sub = 0; sub < SPT; ++sub)
            w_img[(nt * NKD + mt * SPT + sub) * 64 + lane] = EL::from_acc(acc, sub);
    }
    // ---- U~ tile (slice sl, token tile rt): D[token][d_v] = sum_j Tb[token][j] V^T[d_v][j]
    //      stored in the recurrence kernel's accumulator order: [sl][rt][piece][lane], 16 bytes each
    {
        typedef typename EL::UtVec UtVec;
        UtVec* ut = reinterpret_cast<UtVec*>(unit + U::UT_OFF);
        for (int p = wave; p < (DV / 32) * 2; p += 4) {
            const int sl = p % (DV / 32), rt = p / (DV / 32);
            f32x16 acc = {0};
            const float* ar = Lf + (32 * rt + lr) * LF_LD;
            const float* ar10 = Lf + lr * LF_LD + 32;
            const E* br = VTs + (32 * sl + lr) * VT_LD;
            const int ns = (rt == 0) ? NKC / 2 : NKC;
#pragma unroll
            for (int s = 0; s < NKC; ++s)
                if (s < ns) acc = EL::mma(EL::load_scaled((rt == 1 && s < NKC / 2) ? ar10 : ar, bS, s, g), EL::load(br, s, g), acc);
#pragma unroll
            for (int pc = 0; pc < EL::UT_PIECES; ++pc) ut[((sl * 2 + rt) * EL::UT_PIECES + pc) * 64 + lane] = EL::ut_pack(acc, pc);
        }
    }
    // ---- per-token scale factors
    {
        float* aux = reinterpret_cast<float*>(unit + U::AUX_OFF);
        if (tid_p < C) aux[tid_p] = gamS[tid_p];
        else if (tid_p < 2 * C) aux[tid_p] = decS[tid_p - C];
        else if (tid_p == 2 * C) {
            // the chunk's bookkeeping rides along, so the recurrence never waits on a lookup
            int32_t* meta = reinterpret_cast<int32_t*>(aux + 2 * C);
            meta[AUX_EMIT_SLOT] = a.chunk_emit_slot[c];
            meta[AUX_TOK0] = tok0;
            meta[AUX_LEN] = n;
        }
    }
    if (nxt.u >= total) break;
    cur = nxt;
    nxt = locate(cur.u + n_prep_wgs);
    if (!PREFETCH) {
        fetch_kq(cur);
        fetch_v(cur);
    }
    __syncthreads();   // every wave is done with this item's LDS tiles
  }
}

template <typename E, int DK, int DV>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) gdn_prep_kernel(PrepArgs a) {
    const int tid = threadIdx.x;
    const int n_prep_wgs = (int)gridDim.x - a.n_copy_wgs;
    if ((int)blockIdx.x >= n_prep_wgs) {
        // ---- copy role: 16-byte loads over PCIe, four in flight per thread
        const int64_t n4 = a.slot_elems / 4;
        const int64_t step = (int64_t)a.n_copy_wgs * 256;
        for (int st = 0; st < a.n_staged; ++st) {
            const f32x4* src = reinterpret_cast<const f32x4*>(a.host_pool + (int64_t)a.staged_slot[st] * a.host_slot_stride);
            f32x4* dst = reinterpret_cast<f32x4*>(a.staging + (int64_t)st * a.slot_elems);
            int64_t i = (int64_t)((int)blockIdx.x - n_prep_wgs) * 256 + tid;
            for (; i + 3 * step < n4; i += 4 * step) {
                const f32x4 x0 = src[i], x1 = src[i + step], x2 = src[i + 2 * step], x3 = src[i + 3 * step];
                dst[i] = x0; dst[i + step] = x1; dst[i + 2 * step] = x2; dst[i + 3 * step] = x3;
            }
            for (; i < n4; i += step) dst[i] = src[i];
        }
        return;
    }
    prep_body<E, DK, DV>(a, (int)blockIdx.x, n_prep_wgs);
}

}  // namespace gdn
