// Fused throughput kernel (bf16 inputs, d_k = d_v = 128): chunk preparation and recurrence of
// one chain (request, layer, value head) in ONE workgroup, chunk after chunk, the chunk
// operands never leaving the compute unit.
//
// When a call has many more chains than the chip has workgroup slots, the two-kernel path is
// bound by the round trip of the operand image through memory (about three times the
// algorithmic bytes).  Here a workgroup of four waves takes a chain; per chunk it runs the
// preparation (same arithmetic as gdn_prep_kernel: gates, K K^T, K Q^T, T = (I+L)^-1, W, U~)
// with every result kept in LDS or registers, then its four waves, one per 32-column d_v slice,
// run the recurrence step (same arithmetic as gdn_recur_kernel) against those LDS tiles.  HBM
// sees q, k, v, the gates, o and the states, nothing else.  The price: a chain's preparation
// is serial along the chain, so the kernel only pays when chains are plentiful and none is so
// long that it outlasts the rest (the host decides).
//
// LDS plan (76.5 KiB, two workgroups per compute unit):
//   A   K [C][d_k+4]          -> V^T [d_v][C+4] (after K K^T, K Q^T) -> W fragment image (after U~)
//   B   Q [C][d_k+4]          kept until the recurrence has used it
//   KT  K^T [d_k][C+4]        kept until the recurrence has used it
//   LF  L / T fp32 [C][C+4]   T stays fp32; the fp16 fragments of T diag(b) and -T diag(b gam) are made from its rows when used
//   X   P fragment image
//   SM  g, b, gam, dec, -b gam
// The decay to the chunk end is applied to U (a second conversion of U), not to K^T, so that
// the K^T tile serves both W^T = K^T (-T diag(b gam))^T and the state update.
#pragma once
#include "gdn_prep_kernel.h"
#include "gdn_recur_kernel.h"

namespace gdn {

struct FusedArgs {
    const void* q;
    const void* k;
    const void* v;
    const void* beta;
    const void* gate;
    void* o;
    const int32_t* chunk_tok0;
    const int32_t* chunk_len;
    const int32_t* chunk_emit_slot;
    const int32_t* req_chunk_cu;
    const int32_t* req_src_slot;
    const int32_t* req_order;        // requests, longest chain first
    const float* state_src;
    float* state_dst;
    int64_t src_slot_stride, dst_slot_stride;
    int32_t n_chains;
    int32_t L, H_qk, H_v;
    int64_t T_alloc;
    float scale;
    int32_t o_bf16;
};

template <int DK, int DV>
struct FusedSmem {
    static constexpr int C = 64;
    static constexpr int PAD = Elem<half_t>::PAD;
    static constexpr int K_LD = DK + PAD, KT_LD = C + PAD, VT_LD = C + PAD, LF_LD = C + 4;
    static constexpr int a16(int x) { return (x + 15) / 16 * 16; }
    static constexpr int cmax(int x, int y) { return x > y ? x : y; }
    static constexpr int W_IMG_BYTES = 2 * (DK / 16) * 64 * 16;  // W fragments: 2 row tiles x d_k/16 steps
    static constexpr int P_IMG_BYTES = 2 * (C / 16) * 64 * 16;   // P fragments
    static constexpr int A_OFF = 0;
    static constexpr int A_BYTES = cmax(cmax(a16(C * K_LD * 2), a16(DV * VT_LD * 2)), W_IMG_BYTES);
    static constexpr int B_OFF = A_OFF + A_BYTES;
    static constexpr int B_BYTES = a16(C * K_LD * 2);
    static constexpr int KT_OFF = B_OFF + B_BYTES;
    static constexpr int KT_BYTES = a16(DK * KT_LD * 2);
    static constexpr int LF_OFF = KT_OFF + KT_BYTES;
    static constexpr int LF_BYTES = a16(C * LF_LD * 4);
    static constexpr int X_OFF = LF_OFF + LF_BYTES;
    static constexpr int X_BYTES = P_IMG_BYTES;
    static constexpr int SM_OFF = X_OFF + X_BYTES;
    static constexpr int BYTES = SM_OFF + 5 * C * 4;
    static_assert(BYTES <= 80 * 1024, "two workgroups per compute unit");
};

template <int DK, int DV>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) gdn_fused_kernel(FusedArgs a) {
    typedef half_t E;
    typedef Elem<E> EL;
    typedef typename EL::In In;
    typedef typename EL::Frag Frag;
    typedef typename EL::Raw8 Raw8;
    typedef FusedSmem<DK, DV> SM;
    constexpr int C = 64;
    constexpr int K_LD = SM::K_LD, KT_LD = SM::KT_LD, VT_LD = SM::VT_LD, LF_LD = SM::LF_LD;
    constexpr int SPT = EL::STEPS_PER_TILE;
    constexpr int NKD = DK / EL::KSTEP, NKC = C / EL::KSTEP, MT = DK / 32;
    static_assert(DV / 32 == 4 && DK / 32 == 4, "one wave per d_v slice, one W^T row tile per wave");

    extern __shared__ __align__(16) char smem[];
    E* const Ks = reinterpret_cast<E*>(smem + SM::A_OFF);
    E* const VTs = reinterpret_cast<E*>(smem + SM::A_OFF);
    Frag* const w_img = reinterpret_cast<Frag*>(smem + SM::A_OFF);
    E* const Qs = reinterpret_cast<E*>(smem + SM::B_OFF);
    E* const KTs = reinterpret_cast<E*>(smem + SM::KT_OFF);
    float* const Lf = reinterpret_cast<float*>(smem + SM::LF_OFF);
    Frag* const p_img = reinterpret_cast<Frag*>(smem + SM::X_OFF);
    float* const gS = reinterpret_cast<float*>(smem + SM::SM_OFF);
    float* const bS = gS + C;
    float* const gamS = bS + C;
    float* const decS = gamS + C;
    float* const bgS = decS + C;     // -b gam

    const int tid = threadIdx.x;
    const int lane_ = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: say so
    const int lr_ = lane_ & 31;
    const int g_ = lane_ >> 5;
    const int m16_ = lane_ & 15, g4_ = lane_ >> 4;
    const int units = a.L * a.H_v;
    const In* const qg = reinterpret_cast<const In*>(a.q);
    const In* const kg = reinterpret_cast<const In*>(a.k);
    const In* const vg = reinterpret_cast<const In*>(a.v);

    // A thread owns 4-token x 8-column blocks of K, Q and V (256 blocks each at d = 128).
    const int tg_ = tid / (DK / 8), d0_ = (tid % (DK / 8)) * 8;
    const int tgv_ = tid / (DV / 8), d0v_ = (tid % (DV / 8)) * 8;
    static_assert((C / 4) * (DK / 8) == 256 && (C / 4) * (DV / 8) == 256, "one block per thread");

    // ---- the workgroup's items: the chunks of chains blockIdx.x, blockIdx.x + gridDim.x, ...
    struct Item { int chain, c, c_end, lh, tok0, n, eslot; };   // chain < 0: none; eslot: pool slot the chunk's end state goes to, or -1
    auto open_chain = [&](int chain) -> Item {
        Item it;
        for (;; chain += (int)gridDim.x) {
            it.chain = chain < a.n_chains ? chain : -1;
            it.c = it.c_end = it.lh = it.tok0 = it.n = 0;
            it.eslot = -1;
            if (it.chain < 0) return it;
            const int r = a.req_order[chain / units];
            it.lh = chain % units;
            it.c = a.req_chunk_cu[r];
            it.c_end = a.req_chunk_cu[r + 1];
            if (it.c < it.c_end) break;
        }
        it.tok0 = a.chunk_tok0[it.c];
        it.n = a.chunk_len[it.c];
        it.eslot = a.chunk_emit_slot[it.c];
        return it;
    };
    auto next_item = [&](const Item& cur) -> Item {
        if (cur.c + 1 < cur.c_end) {
            Item it = cur;
            it.c = cur.c + 1;
            it.tok0 = a.chunk_tok0[it.c];
            it.n = a.chunk_len[it.c];
            it.eslot = a.chunk_emit_slot[it.c];
            return it;
        }
        return open_chain(cur.chain + (int)gridDim.x);
    };
    Raw8 kraw[4], qraw[4], vraw[4];
    In graw = In(), braw = In();
    auto fetch_kq = [&](const Item& it) {
        const int l = it.lh / a.H_v, hq = (it.lh % a.H_v) / (a.H_v / a.H_qk);
        const int64_t row0 = (int64_t)l * a.T_alloc + it.tok0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = 4 * tg_ + r;
            if (i < it.n) {
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
            if (iv < it.n) vraw[r] = EL::load_raw(vg + ((row0 + iv) * a.H_v + hv) * DV + d0v_);
            else vraw[r] = EL::zero_raw();
        }
        if (wave == 0 && lane_ < it.n) {
            const int64_t gi = (row0 + lane_) * a.H_v + hv;
            graw = reinterpret_cast<const In*>(a.gate)[gi];
            braw = reinterpret_cast<const In*>(a.beta)[gi];
        }
    };

    // The next item's K, Q, V and gates are fetched (raw, into registers) while the current item is
    // processed: 25.0 against 25.8 ms on a 900 k-unit call, 0.84 against 0.91 ms on a 15 k-unit one.
    // This only pays without spills (with 15 to 116 spilled registers the same fetch cost 32 to
    // 39 ms): see the note on opaque lane coordinates in the item loop.  Modes: 0 none, 1 K, Q, V, 2 K, Q.
    constexpr int GDN_FUSED_PREFETCH = 1;
    Item cur = open_chain((int)blockIdx.x);
    if (cur.chain < 0) return;
    if (GDN_FUSED_PREFETCH) fetch_kq(cur);
    if (GDN_FUSED_PREFETCH == 1) fetch_v(cur);
    Item nxt = next_item(cur);

    f32x16 accS[MT];       // this wave's slice of the state: S^T tiles, d_k x 32
    int open = -1;         // chain whose state accS holds
    bool first = true;

    for (;;) {
        // The lane's coordinates are made opaque once per item (and the thread index where it is
        // used): otherwise every address of the unrolled tile accesses below is hoisted out of
        // this loop and held in a register of its own for the whole kernel, which spills (116
        // registers, 2.4 times slower).
        int lane = lane_, lr = lr_, g = g_, m16 = m16_, g4 = g4_, tg = tg_, d0 = d0_, tgv = tgv_, d0v = d0v_;
        pin(lane); pin(lr); pin(g); pin(m16); pin(g4); pin(tg); pin(d0); pin(tgv); pin(d0v);
        const int n = cur.n;
        const int l = cur.lh / a.H_v, hv = cur.lh % a.H_v;
        const int sl = wave;
        const int64_t head_off = ((int64_t)l * a.H_v + hv) * DV * DK + (int64_t)(32 * sl + lr) * DK;

        if (open != cur.chain) {   // a new chain: its start state, from the pool slot or zero
            const int slot = a.req_src_slot[a.req_order[cur.chain / units]];
            if (slot >= 0) {
                load_state<MT>(accS, a.state_src + slot * a.src_slot_stride + head_off, g);
            } else {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) accS[mt][i] = 0.f;
            }
            open = cur.chain;
        }
        if (!first) __syncthreads();   // the previous item's recurrence is done with every LDS tile
        first = false;

        if (!GDN_FUSED_PREFETCH) fetch_kq(cur);
        if (GDN_FUSED_PREFETCH != 1) fetch_v(cur);   // V and the gates: used two barriers from here
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
        // ---- stage K, Q (row-major) and K^T (token-contiguous) as fp16
        {
            float kv[4][8];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = 4 * tg + r;
                float qv[8];
                EL::unpack(kraw[r], kv[r]);
                EL::unpack(qraw[r], qv);
                EL::store4(Ks + i * K_LD + d0, kv[r][0], kv[r][1], kv[r][2], kv[r][3]);
                EL::store4(Ks + i * K_LD + d0 + 4, kv[r][4], kv[r][5], kv[r][6], kv[r][7]);
                EL::store4(Qs + i * K_LD + d0, qv[0], qv[1], qv[2], qv[3]);
                EL::store4(Qs + i * K_LD + d0 + 4, qv[4], qv[5], qv[6], qv[7]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
                EL::store4(KTs + (d0 + e) * KT_LD + 4 * tg, kv[0][e], kv[1][e], kv[2][e], kv[3][e]);
        }
        if (GDN_FUSED_PREFETCH && nxt.chain >= 0) fetch_kq(nxt);
        __syncthreads();

        // ---- K K^T -> L (fp32) and K Q^T -> P fragments (to X: the previous chunk's recurrence is done with it)
        //      wave 0: KK(0,0) KQ(0,0)   wave 1: KK(1,0)   wave 2: KK(1,1) KQ(1,1)   wave 3: KQ(0,1)
        int p_mj = -1, p_ni = -1;
        {
            int kk_mi = -1, kk_nj = -1;
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
                f32x16 acc = {0};
                const E* ar = Ks + (32 * p_mj + lr) * K_LD;   // rows: key token j
                const E* br = Qs + (32 * p_ni + lr) * K_LD;   // rows: query token i
#pragma unroll
                for (int s = 0; s < NKD; ++s) acc = EL::mma(EL::load(ar, s, g), EL::load(br, s, g), acc);
                const int i = 32 * p_ni + lr;
                const float gi = gS[i];
#pragma unroll
                for (int idx = 0; idx < 16; ++idx) {
                    const int j = 32 * p_mj + acc_row(idx, g);
                    const float val = a.scale * EL::exp_(fminf(gi - gS[j], 0.f)) * acc[idx];
                    acc[idx] = (j <= i) ? val : 0.f;
                }
#pragma unroll
                for (int sub = 0; sub < SPT; ++sub) p_img[(p_ni * NKC + p_mj * SPT + sub) * 64 + lane] = EL::from_acc(acc, sub);
            }
        }
        __syncthreads();  // L is complete; K in LDS is dead

        // ---- V^T into K's place
        {
            float vv[4][8];
#pragma unroll
            for (int r = 0; r < 4; ++r) EL::unpack(vraw[r], vv[r]);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                EL::store4(VTs + (d0v + e) * VT_LD + 4 * tgv, vv[0][e], vv[1][e], vv[2][e], vv[3][e]);
        }
        if (GDN_FUSED_PREFETCH == 1 && nxt.chain >= 0) fetch_v(nxt);

        // ---- T = (I + L)^-1, fp32, by 16x16 blocks (see gdn_prep_kernel).  Stage 1: diagonal blocks
        //      by (I + D)^-1 = (I + D^8)(I + D^4)(I + D^2)(I - D), in registers.
        {
            float* const D = Lf + (16 * wave) * LF_LD + 16 * wave;
            const f32x4 y = inv16_unit_lower<LF_LD>(D, m16, g4);
#pragma unroll
            for (int e = 0; e < 4; ++e) D[(4 * g4 + e) * LF_LD + m16] = y[e];
        }
        __syncthreads();  // diagonal blocks of T in place
        auto blk = [&](int br, int bc) -> const float* { return Lf + (16 * br) * LF_LD + 16 * bc; };
        if (wave < 2) {   // Stage 2: T_10 = -T_11 (L_10 T_00), T_32 = -T_33 (L_32 T_22)
            const int ra = 2 * wave + 1, rb = 2 * wave;
            f32x4 m = {0, 0, 0, 0};
            m = mm16_ll<LF_LD>(m, blk(ra, rb), blk(rb, rb), m16, g4);
            f32x4 r = {0, 0, 0, 0};
            r = mm16_lr<LF_LD>(r, blk(ra, ra), m, m16, g4);
#pragma unroll
            for (int e = 0; e < 4; ++e) Lf[(16 * ra + 4 * g4 + e) * LF_LD + 16 * rb + m16] = -r[e];
        }
        __syncthreads();
        {   // Stage 3: the 32x32 block below the diagonal; wave w owns T_ab, a = 2 + w/2, b = w%2
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

        // ---- T stays in fp32: the operand fragments of T diag(b) and -T diag(b gam) are made from its
        //      rows on the fly (two 16-byte reads, the scale, the conversion), so no fp16 copy of T is
        //      written and no barrier separates T from its two uses.  Entries above the diagonal inside
        //      the tiles that are read are exact zeros (written so by the K K^T epilogue and kept by the
        //      inversion); the tile above the diagonal tiles holds the block below them.

        // ---- U~ for this wave's slice (both token tiles), straight into the recurrence's accumulators
        f32x16 accU[2];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            f32x16 acc = {0};
            const float* ar = Lf + (32 * rt + lr) * LF_LD;
            const float* ar10 = Lf + lr * LF_LD + 32;   // rows 32.., columns 0..31 of T live above the diagonal tiles
            const E* br = VTs + (32 * sl + lr) * VT_LD;
#pragma unroll
            for (int s = 0; s < NKC; ++s)
                if (s < (rt == 0 ? NKC / 2 : NKC))
                    acc = EL::mma(EL::load_scaled((rt == 1 && s < NKC / 2) ? ar10 : ar, bS, s, g), EL::load(br, s, g), acc);
            accU[rt] = acc;
        }
        __syncthreads();  // V^T is dead

        // ---- W^T tiles (d_k rows 32 wave .., both token tiles) -> W fragments in A
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int mt = wave;
            f32x16 acc = {0};
            const E* ar = KTs + (32 * mt + lr) * KT_LD;
            const float* br = Lf + (32 * nt + lr) * LF_LD;
            const float* br10 = Lf + lr * LF_LD + 32;
#pragma unroll
            for (int s = 0; s < NKC; ++s)
                if (s < (nt == 0 ? NKC / 2 : NKC))
                    acc = EL::mma(EL::load(ar, s, g), EL::load_scaled((nt == 1 && s < NKC / 2) ? br10 : br, bgS, s, g), acc);
#pragma unroll
            for (int sub = 0; sub < SPT; ++sub) w_img[(nt * NKD + mt * SPT + sub) * 64 + lane] = EL::from_acc(acc, sub);
        }
        __syncthreads();  // W image complete

        // ---- recurrence step of this chunk, slice sl = wave (see gdn_recur_kernel)
        {
            Frag sf[NKD];
#pragma unroll
            for (int s = 0; s < NKD; ++s) sf[s] = EL::from_acc(accS[s / SPT], s % SPT);
            // U = U~ + W S^T
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int s = 0; s < NKD; ++s) accU[rt] = EL::mma(w_img[(rt * NKD + s) * 64 + lane], sf[s], accU[rt]);
            Frag uf[2 * SPT];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int s = 0; s < SPT; ++s) uf[rt * SPT + s] = EL::from_acc(accU[rt], s);
            // O^T = (S Q^T) diag(gam) + U^T P^T with the state of the chunk start
            const int64_t row0 = (int64_t)l * a.T_alloc + cur.tok0;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                f32x16 acc = {0};
                const E* qr = Qs + (32 * tt + lr) * K_LD;
#pragma unroll
                for (int s = 0; s < NKD; ++s) acc = EL::mma(sf[s], EL::load(qr, s, g), acc);
                const float gm = gamS[32 * tt + lr] * a.scale;
#pragma unroll
                for (int k = 0; k < 16; ++k) acc[k] *= gm;
#pragma unroll
                for (int s = 0; s < (tt + 1) * SPT; ++s) acc = EL::mma(uf[s], p_img[(tt * NKC + s) * 64 + lane], acc);
                store_o_tile<DV>(a, row0, hv, sl, lr, g, n, tt, acc);
            }
            // state update: S^T = gam_C S^T + sum_j K^T[.][j] (dec_j U[j][.])
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const f32x4 dc = *reinterpret_cast<const f32x4*>(decS + 32 * rt + 8 * b + 4 * g);
#pragma unroll
                    for (int e = 0; e < 4; ++e) accU[rt][4 * b + e] *= dc[e];
                }
#pragma unroll
                for (int s = 0; s < SPT; ++s) uf[rt * SPT + s] = EL::from_acc(accU[rt], s);
            }
            const float gam_last = gamS[C - 1];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int i = 0; i < 16; ++i) accS[mt][i] *= gam_last;
                const E* kr = KTs + (32 * mt + lr) * KT_LD;
#pragma unroll
                for (int s = 0; s < NKC; ++s) accS[mt] = EL::mma(EL::load(kr, s, g), uf[s], accS[mt]);
            }
            // checkpoint emission: exact state after the last token of this chunk
            const int eslot = cur.eslot;   // looked up one item ahead, with the chunk's other bookkeeping
            if (eslot >= 0) store_state<MT>(accS, a.state_dst + eslot * a.dst_slot_stride + head_off, g);
        }

        if (nxt.chain < 0) break;
        cur = nxt;
        nxt = next_item(cur);
    }
}

}  // namespace gdn
