// Fused throughput kernel (bf16 inputs, d_k = d_v = D = 128 or 64): chunk preparation and recurrence of
// one chain (request, layer, value head) in ONE workgroup, chunk after chunk, the chunk
// operands never leaving the compute unit.  HBM sees q, k, v, the gates, o and the states,
// nothing else.  A chain's chunks are serial, so the kernel only pays when chains are plentiful
// and none is so long that it outlasts the rest (the host decides).  The grid is persistent (one to three workgroups per
// compute unit); the chains come longest first and are taken in turn by whichever workgroup is free (see the items).
//
// Per 64-token chunk, with g the running sum of log a, gam = exp(g), L_ij = b_i exp(g_i - g_j)(k_i.k_j)
// for j < i, the chunk-local form of the gated delta rule is
//     (I + L) U = diag(b) V - diag(b gam) K S0^T ,   O = diag(gam scale) Q S0^T + P U ,
//     S_C = gam_C S0 + (diag(dec) U)^T K ,           P_ij = scale exp(g_i - g_j)(q_i.k_j), j <= i, dec_i = exp(g_C - g_i).
// T = (I + L)^-1 is never formed.  The chunk is cut into four blocks of 16 tokens and U is found by block
// forward substitution, block row a after block row a-1:
//     U_a = T_aa diag(b_a) V_a  -  T_aa diag(b gam)_a (K_a S0^T)  -  sum_{c<a} (T_aa L_ac) U_c ,
// where only the four 16x16 diagonal inverses T_aa = (I + L_aa)^-1 are computed (fp32, in registers, see
// inv16_tiles) and the state-independent blocks  T_aa diag(b),  -T_aa diag(b gam),  -T_aa L_ac  (fp32 products,
// rounded once to fp16) are left in LDS as matrix-core operands.  Every other product is a
// v_mfma_f32_16x16x32_f16, a lone 16-row block being paired with a zero half (one instruction shape throughout: a
// 16x16x16 that takes as its accumulator input the result of the 16x16x32 issued just before it was seen to read
// stale values).  An accumulator tile holds rows 4 g4 + e of column m in lane (m, g4), which is exactly the B
// operand of a product that contracts over those rows, so K S0^T, U_c and U feed the next product from registers.
//
// A workgroup is four waves.  Preparation: wave a owns block row a (its diagonal inverse, its L blocks and
// their products with T_aa) and the P blocks of query block 3 - a, five 16x16 gram blocks each.  Recurrence:
// wave w owns the D / 4 d_v columns of the state from (D / 4) w on (D / 64 16-column tiles, the state of a tile in
// D / 16 accumulator tiles over d_k); the state products of block row a + 1 are issued ahead of block row a's
// substitution.  Three barriers per chunk.  The rows of the next chunk are fetched into registers meanwhile, in three
// instalments spread over the staging and the preparation (see the staging loop).
//
// Grouped value heads (GV = 2): two value heads of one query/key head in a workgroup of eight waves, four per head as
// above.  K and Q are fetched (waves 0-3: K, waves 4-7: Q), converted and held in LDS once for both; each head has its own
// V tile, pair tiles, gate vectors and state, and its arithmetic is that of the one-head kernel instruction for instruction.
// The barriers span all eight waves.
//
// LDS (FusedSmem<D, GV>: 73 KB at D = 128, two workgroups per compute unit; 49 KB at D = 64, three; a pair 113 KB / 81 KB, one):
//   K, Q, V  fp16 [64][D], rows unpadded, the 16-byte pieces of a row XOR-swizzled with the row number (swz):
//            row reads (lane = token, one piece: the A/B operand of a product over d_k) are free of bank
//            conflicts, transposing reads (ds_read_b64_tr_b16: lane = column, four tokens: K^T for the state
//            update, V^T for the substitution) touch one half of every piece and are two-way at best
//   pair tiles [16][2 x 16 (+8)] fp16, two blocks side by side so that a 16x16x32 operand is one 16-byte read:
//            TbTg[a] = [T_aa diag(b) | -T_aa diag(b gam)],  M = -T_aa L_ac (c < a),  P (c <= ia); a lone block's
//            partner half stays zero from the start of the kernel
//   Tf[w]    fp32 [16][20]: a wave's T_aa on its way from the accumulator layout to its transpose
//   g, b, gam, dec, and the factors of the decay between blocks (s, r_c; see the gates): fp32 [64] each
//   one word: the chain the workgroup holds in reserve, on its way from the wave that drew it to the others
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
    int32_t* next_chain;             // one word, zero when the kernel starts: chains handed out beyond the first two rounds
    const float* state_src;
    float* state_dst;
    int64_t src_slot_stride, dst_slot_stride;
    int32_t n_chains;
    int32_t L, H_qk, H_v;
    int64_t T_alloc;
    float scale;
    int32_t o_bf16;
};

// GV value heads of one query/key head share a workgroup (GV x 4 waves) and its K and Q tiles; everything that depends on
// the value head (V, the pair tiles, Tf, the gate vectors) exists once per head, HEAD_BYTES apart.
template <int D_, int GV_ = 1>
struct FusedSmem {
    static constexpr int C = 64, D = D_, GV = GV_;
    static constexpr int TILE_BYTES = C * D * 2;            // one of K, Q, V
    static constexpr int PAIR_LD = 40, TF_LD = 20;          // halfs / floats per row
    static constexpr int PAIR_BYTES = 16 * PAIR_LD * 2;     // one 16 x (2 x 16) fp16 pair tile
    static constexpr int K_OFF = 0;
    static constexpr int Q_OFF = K_OFF + TILE_BYTES;
    static constexpr int V_OFF = Q_OFF + TILE_BYTES;         // V of head h at V_OFF + h TILE_BYTES
    static constexpr int HEAD_OFF = V_OFF + GV * TILE_BYTES; // the per-head part of head h at HEAD_OFF + h HEAD_BYTES, offsets inside it:
    static constexpr int TBTG_OFF = 0;                       // pair tile a: [T_aa diag(b) | -T_aa diag(b gam)]
    static constexpr int M_OFF = TBTG_OFF + 4 * PAIR_BYTES;  // pair tiles (1: M10,0) (2: M20,M21) (3: M30,M31) (3: M32,0)
    static constexpr int P_OFF = M_OFF + 4 * PAIR_BYTES;     // pair tiles (0: P00,0) (1: P10,P11) (2: P20,P21) (2: P22,0) (3: P30,P31) (3: P32,P33)
    static constexpr int TF_OFF = P_OFF + 6 * PAIR_BYTES;
    static constexpr int SM_OFF = TF_OFF + 4 * 16 * TF_LD * 4;
    static constexpr int HEAD_BYTES = SM_OFF + 8 * C * 4;    // g, b, gam, dec, s, 3 x r
    static constexpr int RESERVE_OFF = HEAD_OFF + GV * HEAD_BYTES;   // one word: the chain the workgroup opens after the next one
    static constexpr int BYTES = RESERVE_OFF + 16;
    static_assert(HEAD_OFF % 16 == 0 && HEAD_BYTES % 16 == 0 && M_OFF % 16 == 0 && P_OFF % 16 == 0 && TF_OFF % 16 == 0 && SM_OFF % 16 == 0, "alignment");
    static_assert(GV == 1 || GV == 2, "one head or a pair");
    static_assert(GV == 2 ? BYTES <= 160 * 1024 : BYTES <= 80 * 1024, "a pair has a compute unit to itself; two single-head workgroups share one");
    // pair tile index of block (a, c) of M (c < a) and of P (c <= a)
    static constexpr __host__ __device__ int m_pair(int a, int c) { return (a == 1 ? 0 : a == 2 ? 1 : 2) + (c >> 1); }
    static constexpr __host__ __device__ int p_pair(int a, int c) { return (a == 0 ? 0 : a == 1 ? 1 : a == 2 ? 2 : 4) + (c >> 1); }
};

// A wave-uniform word of the call's plan, read through the scalar cache (the plan is read-only while the kernel runs).
// A vector load here would share the in-flight counter of the output stores and make the item loop wait for them.
__device__ __forceinline__ int32_t plan_word(const int32_t* p, int i) {
    typedef const __attribute__((address_space(4))) int32_t* cptr;
    return ((cptr)(uintptr_t)p)[i];
}

typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;

// Swizzle of the 16-byte pieces of a row of a [64][D] fp16 tile: piece p of row r sits at p ^ swz(r).  The LDS has 64
// banks of 4 bytes.  D = 128 (a row is 256 bytes, so without it every row starts at bank 0): swz is a bijection of the low
// four bits of the row: 16 lanes reading the same piece of 16 consecutive rows (row reads, 16 bytes per lane) touch 16
// different bank groups; its bit 3 also moves with the row's bit 0, so that the 8 rows x 4 pieces a transposing read
// addresses per cycle (8 bytes per lane, the same half of every piece) spread two by two over all 16 groups, which is the
// best that half-pieces allow.  D = 64 (128-byte rows, two to a bank span, eight pieces): the row's bits 1..3, so that 16
// consecutive rows with the same piece again touch 16 different groups.  Either way swz(r + 16) = swz(r).
template <int D>
__device__ __forceinline__ int swz(int row) { return D == 128 ? ((row & 15) ^ ((row & 1) << 3)) : ((row >> 1) & 7); }

__device__ __forceinline__ half4 cvt4(const f32x4& x) {
    half4 h;
    h[0] = (half_t)x[0]; h[1] = (half_t)x[1]; h[2] = (half_t)x[2]; h[3] = (half_t)x[3];
    return h;
}
__device__ __forceinline__ half8 cat8(const half4& lo, const half4& hi) {
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
__device__ __forceinline__ f32x4 mma32(const half8& a, const half8& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ half4 tr_read(const char* p) {
    return __builtin_bit_cast(half4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p)));
}

// (I + D)^-1 of a strictly lower triangular 16x16 block given the accumulator-layout tiles of D (d: element e of
// lane (m, g4) is D[4 g4 + e][m]) and of its transpose (dt: D[m][4 g4 + e]); the nilpotent product of
// inv16_unit_lower, all in registers.  Returns the tile of the inverse.
__device__ __forceinline__ f32x4 inv16_tiles(const f32x4& d, const f32x4& dt, int m, int g4) {
    f32x4 y;
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = ((4 * g4 + e) == m ? 1.f : 0.f) - d[e];
    const f32x4 zero = {0, 0, 0, 0};
    const f32x4 p2 = mm16_rr(zero, dt, d), p2t = mm16_rr(zero, d, dt);
    y = mm16_rr(y, p2t, y);
    const f32x4 p4 = mm16_rr(zero, p2t, p2), p4t = mm16_rr(zero, p2, p2t);
    y = mm16_rr(y, p4t, y);
    const f32x4 p8t = mm16_rr(zero, p4, p4t);
    return mm16_rr(y, p8t, y);
}

// Profiling build only (-DGDN_PHASE_STAMPS, a library of its own: see build.py): cycle stamps at the phase boundaries of
// the 40th item of every eighth workgroup (the kernel's steady state), one set per wave, read back by gdn_phase_stamps.  The product build has none.
#ifdef GDN_PHASE_STAMPS
__device__ unsigned long long g_phase_ts[64 * 4 * 16];
#define GDN_PHASE(k_)                                                                                   \
    do {                                                                                                \
        if (gdn_item == 40 && (blockIdx.x & 7) == 0 && blockIdx.x < 512 && lane_ == 0 && hsel == 0)     \
            g_phase_ts[((blockIdx.x >> 3) * 4 + wave) * 16 + (k_)] = __builtin_readcyclecounter();      \
    } while (0)
#define GDN_PHASE_ITEM() (++gdn_item)
#else
#define GDN_PHASE(k_) do {} while (0)
#define GDN_PHASE_ITEM() ((void)0)
#endif

template <bool O_BF16, int D, int GV>
__global__ void __launch_bounds__(256 * GV) __attribute__((amdgpu_waves_per_eu(2, (D == 128 || GV == 2) ? 2 : 3))) gdn_fused_kernel(FusedArgs a) {
    typedef Elem<half_t> EL;
    typedef EL::In In;
    typedef EL::Raw8 Raw8;
    typedef FusedSmem<D, GV> SM;
    constexpr int C = 64, DK = D, DV = D, PLD = SM::PAIR_LD;
    constexpr int NT = D / 64;        // 16-column tiles of the state per wave (a wave owns D / 4 columns of d_v)
    constexpr int SS = D / 32;        // steps of 32 over d_k (one 16-byte piece per lane and step)
    constexpr int MT = D / 16;        // 16-wide tiles over d_k
    constexpr int RBY = 2 * D;        // bytes of a K, Q or V tile row
    constexpr int PCS = D / 8;        // 16-byte pieces per row
    constexpr int ROWS = D / 32;      // rows of each tensor a thread stages (256 threads, 64 rows of PCS pieces)
    constexpr int WC = D / 4;         // d_v columns per wave

    // A workgroup is GV groups of four waves, group hsel on value head hsel of the workgroup's GV heads (which share a
    // query/key head: the host sees to that); wave = the wave's number inside its group.
    const int tid = threadIdx.x & 255;
    const int lane_ = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: say so
    const int hsel = GV == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8);

    extern __shared__ __align__(16) char smem[];
    char* const Kt = smem + SM::K_OFF;
    char* const Qt = smem + SM::Q_OFF;
    char* const Vt = smem + SM::V_OFF + hsel * SM::TILE_BYTES;
    char* const hsm = smem + SM::HEAD_OFF + hsel * SM::HEAD_BYTES;
    half_t* const tbtg = reinterpret_cast<half_t*>(hsm + SM::TBTG_OFF);
    half_t* const mimg = reinterpret_cast<half_t*>(hsm + SM::M_OFF);
    half_t* const pimg = reinterpret_cast<half_t*>(hsm + SM::P_OFF);
    float* const gS = reinterpret_cast<float*>(hsm + SM::SM_OFF);
    float* const bS = gS + C;
    float* const gamS = bS + C;
    float* const decS = gamS + C;
    float* const sS = decS + C;      // s_j = exp(g_end(block of j) - g_j)
    float* const rS = sS + C;        // [3][64]: r_i(c) = exp(g_i - g_end(c)), c = 0..2, for tokens i of later blocks

    float* const Tf = reinterpret_cast<float*>(hsm + SM::TF_OFF) + wave * 16 * SM::TF_LD;
    const int units = a.L * a.H_v / GV;     // chains of a request: one per layer and group of GV value heads
    const In* const qg = reinterpret_cast<const In*>(a.q);
    const In* const kg = reinterpret_cast<const In*>(a.k);
    const In* const vg = reinterpret_cast<const In*>(a.v);

    // A thread owns ROWS-token x 8-column blocks (256 blocks per tensor): of K, Q and V when the workgroup has one head; of
    // its head's V and of one of the shared tensors (group 0: K, group 1: Q) when it has two.
    const int tg_ = tid / PCS, d0_ = (tid % PCS) * 8;

    // The unused halves of the pair tiles (a lone block is paired with zeros) are zeroed once; nothing writes them later.
    for (int i = tid; i < (SM::TF_OFF - SM::TBTG_OFF) / 16; i += 256)
        reinterpret_cast<u32x4*>(hsm + SM::TBTG_OFF)[i] = u32x4{0u, 0u, 0u, 0u};

    // ---- the workgroup's items: the chunks of one chain after the other.  The chains come longest first (every one has
    //      at least one chunk: requests without tokens are not among them).  Workgroup b starts with chain b and holds chain
    //      2 gridDim.x - 1 - b in reserve (the second round dealt backwards: the longest chain of the first round is followed by
    //      the shortest of the second); from then on a workgroup that opens its reserve draws a new one from a counter in memory
    //      (2 gridDim.x + the counter's value: longest-first list scheduling, so a workgroup that drew short chains simply draws
    //      more of them).  The draw is an atomic with a round trip to memory, so it is made a whole item before its result
    //      can be needed: the first wave issues it when the reserve is opened, puts the result into LDS after the next wait
    //      on its memory operations, and every wave picks it up behind the barrier at the top of the next item.  Which
    //      workgroup runs a chain does not touch the chain's arithmetic: results are the same bit for bit whatever the draw.
    struct Item { int chain, c, c_end, lh, tok0, n, eslot; };   // chain < 0: none; eslot: pool slot the chunk's end state goes to, or -1
    int* const reserve_lds = reinterpret_cast<int*>(smem + SM::RESERVE_OFF);
    int reserve = 2 * (int)gridDim.x - 1 - (int)blockIdx.x;   // the chain to open after the current one
    bool reserve_stale = false;                       // opened: the next one is on its way through LDS
    bool draw_pending = false;                        // first wave: an atomic is in flight
    int drawn = 0;                                    // first wave, lane 0: its result
    auto open_chain = [&](int chain) -> Item {
        Item it;
        it.chain = chain < a.n_chains ? chain : -1;
        it.c = it.c_end = it.lh = it.tok0 = it.n = 0;
        it.eslot = -1;
        if (it.chain < 0) return it;
        const int r = plan_word(a.req_order, chain / units);
        it.lh = (chain % units) * GV + hsel;
        it.c = plan_word(a.req_chunk_cu, r);
        it.c_end = plan_word(a.req_chunk_cu, r + 1);
        it.tok0 = plan_word(a.chunk_tok0, it.c);
        it.n = plan_word(a.chunk_len, it.c);
        it.eslot = plan_word(a.chunk_emit_slot, it.c);
        return it;
    };
    auto next_item = [&](const Item& cur) -> Item {
        if (cur.c + 1 < cur.c_end) {
            Item it = cur;
            it.c = cur.c + 1;
            it.tok0 = plan_word(a.chunk_tok0, it.c);
            it.n = plan_word(a.chunk_len, it.c);
            it.eslot = plan_word(a.chunk_emit_slot, it.c);
            return it;
        }
        const Item it = open_chain(reserve);
        if (it.chain >= 0) {       // the reserve is used up: draw the next one (past the last chain nothing is left to draw)
            if (wave == 0 && hsel == 0 && lane_ == 0)
                drawn = 2 * (int)gridDim.x + __hip_atomic_fetch_add(a.next_chain, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            draw_pending = true;
            reserve_stale = true;
        }
        return it;
    };
    // The next item's K, Q, V and gates are fetched (raw, into registers) while the current item is processed.
    Raw8 kraw[ROWS], qraw[ROWS], vraw[ROWS];   // two heads: kraw holds the group's shared tensor, qraw is unused
    In graw = In();      // wave 0: the lane's gate; wave 1: its beta
    // Buffer loads: a wave-uniform descriptor per tensor that starts at the chunk's first row of this head and ends with its
    // last row (rows past n, and every row when there is no item, read as zeros, no branch), 32-bit per-lane offsets.  Read
    // once, never again: non-temporal.  (Written out as macros: descriptors do not pass through lambdas on the host pass.)
    const int qk_step = a.H_qk * DK * 2, v_step = a.H_v * DV * 2;      // bytes from token to token
    const In* const kg_ = (GV == 2 && hsel == 1) ? qg : kg;            // the group's shared tensor
#define GDN_FETCH_DESCRIPTORS(it_)                                                                                              \
    const int f_l = (it_).lh / a.H_v, f_hv = (it_).lh % a.H_v, f_hq = f_hv / (a.H_v / a.H_qk);                                 \
    const int64_t f_row0 = (int64_t)f_l * a.T_alloc + (it_).tok0;                                                               \
    const bool f_on = (it_).chain >= 0;                                                                                         \
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(const_cast<In*>(kg_ + (f_row0 * a.H_qk + f_hq) * DK), 0, \
                                                                         f_on ? ((it_).n - 1) * qk_step + DK * 2 : 0, 0x00020000); \
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<In*>(qg + (f_row0 * a.H_qk + f_hq) * DK), 0,  \
                                                                         f_on ? ((it_).n - 1) * qk_step + DK * 2 : 0, 0x00020000); \
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(const_cast<In*>(vg + (f_row0 * a.H_v + f_hv) * DV), 0,   \
                                                                         f_on ? ((it_).n - 1) * v_step + DV * 2 : 0, 0x00020000)
#define GDN_FETCH_K(r_, tg_v, d0_v) kraw[r_] = __builtin_bit_cast(Raw8, __builtin_amdgcn_raw_buffer_load_b128(rk, (ROWS * (tg_v) + (r_)) * qk_step + (d0_v) * 2, 0, 2))
#define GDN_FETCH_Q(r_, tg_v, d0_v) if (GV == 1) qraw[r_] = __builtin_bit_cast(Raw8, __builtin_amdgcn_raw_buffer_load_b128(rq, (ROWS * (tg_v) + (r_)) * qk_step + (d0_v) * 2, 0, 2))
#define GDN_FETCH_V(r_, tg_v, d0_v) vraw[r_] = __builtin_bit_cast(Raw8, __builtin_amdgcn_raw_buffer_load_b128(rv, (ROWS * (tg_v) + (r_)) * v_step + (d0_v) * 2, 0, 2))
// All ROWS rows of one tensor, pinned where they stand: the compiler would otherwise gather the loads into one burst again.
#define GDN_FETCH_ALL(which_, tg_v, d0_v)                                                                                        \
    do {                                                                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                                                      \
        _Pragma("unroll") for (int r_ = 0; r_ < ROWS; ++r_) { which_(r_, tg_v, d0_v); }                                        \
        __builtin_amdgcn_sched_barrier(0);                                                                                      \
    } while (0)
    // The 64 gates are read by wave 0 and the 64 betas by wave 1 only: a lane per token, 2 bytes each at a stride of a
    // token's heads, is 64 separate memory requests per instruction.
#define GDN_FETCH_GATES(it_, lane_v)                                                                                             \
    do {                                                                                                                        \
        if ((lane_v) < (it_).n && wave < 2 && f_on)                                                                             \
            graw = (reinterpret_cast<const In*>(wave == 0 ? a.gate : a.beta) + (f_row0 * a.H_v + f_hv))[(lane_v) * a.H_v];      \
    } while (0)

    Item cur = open_chain((int)blockIdx.x);
    if (cur.chain < 0) return;
    {
        GDN_FETCH_DESCRIPTORS(cur);
        GDN_FETCH_ALL(GDN_FETCH_K, tg_, d0_);
        GDN_FETCH_ALL(GDN_FETCH_Q, tg_, d0_);
        GDN_FETCH_ALL(GDN_FETCH_V, tg_, d0_);
        GDN_FETCH_GATES(cur, lane_);
    }
    wait_vmcnt<0>();   // the first item's inputs: inside the loop the fetched registers are then known to have landed on every path

    // State tile (mt = 2 s + h, nt): element e of lane (m, g4) is S[32 w + 16 nt + m][32 s + 8 g4 + 4 h + e], so that the
    // tile pair of step s is, lane for lane, the operand over d_k columns 32 s + 8 g4 .. + 7: one 16-byte piece of a K or Q row.
    f32x4 accS[MT][NT];
    int open = -1;         // chain whose state accS holds
    bool first = true;
    bool state_pending = false;   // the start state of a new chain is still on its way

    int gdn_item = 0;      // items done (used by the profiling build only)
    (void)gdn_item;
    for (;;) {
        // The lane's coordinates are made opaque once per item: otherwise every address of the unrolled tile
        // accesses below is hoisted out of this loop and held in a register of its own for the whole kernel.
        int lane = lane_, tg = tg_, d0 = d0_;
        pin(lane); pin(tg); pin(d0);
        const int m = lane & 15, g4 = lane >> 4;
        const int n = cur.n;
        const int l = cur.lh / a.H_v, hv = cur.lh % a.H_v;
        const int64_t head_off = ((int64_t)l * a.H_v + hv) * DV * DK;
        // LDS byte offsets of this lane inside a K/Q/V tile; the rest of every address is a compile-time constant.
        //   row reads: lane (m, g4) reads piece 4 s + g4 of row 16 blk + m, which sits at (4 s + g4) ^ swz(m)
        int row_b[SS], tr_b[SS];
#pragma unroll
        for (int s = 0; s < SS; ++s) row_b[s] = m * RBY + 16 * ((4 * s + g4) ^ swz<D>(m));     // + blk * 16 * RBY
        //   transposing reads of K for the state update: lane j of group g4 addresses token tok0 + 4 g4 + j / 4, d_k columns
        //   32 s + 8 (j % 4) + 4 h ...: lane i then receives column 32 s + 8 (i / 4) + 4 h + i % 4, which is row i of state tile 2 s + h
        const int trow = 4 * g4 + (m >> 2);
#pragma unroll
        for (int s = 0; s < SS; ++s) tr_b[s] = trow * RBY + 16 * ((4 * s + (m & 3)) ^ swz<D>(trow));   // + tok0 * RBY + 8 h
        //   transposing reads of V for the substitution: lane i receives column 32 w + 16 nt + i: lane j addresses columns
        //   32 w + 16 nt + 4 (j % 4) ..., i.e. piece 4 w + 2 nt + (j % 4) / 2, half (j % 4) % 2
        int tv[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            tv[nt] = trow * RBY + 16 * (((WC / 8) * wave + 2 * nt + ((m & 3) >> 1)) ^ swz<D>(trow)) + 8 * (m & 1);   // + tok0 * RBY

        if (open != cur.chain) {   // a new chain: its start state, from the pool slot or zero
            const int slot = plan_word(a.req_src_slot, plan_word(a.req_order, cur.chain / units));
            if (slot >= 0) {
                const float* src = a.state_src + slot * a.src_slot_stride + head_off;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        accS[mt][nt] = *reinterpret_cast<const f32x4*>(src + (WC * wave + 16 * nt + m) * DK + 32 * (mt >> 1) + 8 * g4 + 4 * (mt & 1));
                // not waited for here: the first chunk's gates, staging and preparation do not need the state, and the
                // recurrence waits below
                state_pending = true;
            } else {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) accS[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            open = cur.chain;
        }
        if (!first) __syncthreads();   // the previous item's recurrence is done with every LDS tile
        first = false;
        if (reserve_stale) {           // the chain drawn during the previous item, now in LDS for every wave
            reserve = __builtin_amdgcn_readfirstlane(reserve_lds[0]);
            reserve_stale = false;
        }
        const Item nxt = next_item(cur);
        GDN_PHASE_ITEM();
        GDN_PHASE(0);

        // ---- gates, by wave 0: g_i = inclusive running sum of log a and what derives from it; identity beyond n.  Between
        //      blocks of 16 tokens the decay factors into a row and a column part, exp(g_i - g_j) = exp(g_i - g_end(c))
        //      exp(g_end(c) - g_j) for j in block c and i in a later block, both exponents <= 0 since g never rises: the
        //      blocks off the diagonal then need no exponential per element.  Wave 1 stores the betas.
        if (wave == 0) {
            const float la = lane < n ? fmaxf(EL::log_(EL::widen(graw)), -88.f) : 0.f;
            const float s = wave_running_sum(la);
            const int sbits = __builtin_bit_cast(int, s);
            const float e0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(sbits, 15));
            const float e1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(sbits, 31));
            const float e2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(sbits, 47));
            const float g_last = wave_last_lane(s);
            const float eb = lane < 16 ? e0 : lane < 32 ? e1 : lane < 48 ? e2 : g_last;
            gS[lane] = s;
            gamS[lane] = EL::exp_(s);
            decS[lane] = EL::exp_(g_last - s);
            sS[lane] = EL::exp_(fminf(eb - s, 0.f));
            rS[lane] = EL::exp_(fminf(s - e0, 0.f));
            rS[C + lane] = EL::exp_(fminf(s - e1, 0.f));
            rS[2 * C + lane] = EL::exp_(fminf(s - e2, 0.f));
        } else if (wave == 1) {
            bS[lane] = lane < n ? EL::widen(graw) : 0.f;
        }
        // ---- stage K, Q, V as fp16 (exact widening of bf16): one 16-byte piece per row and tensor, swizzled
        //      The next item's rows are fetched in three instalments, each where the registers it overwrites are free and
        //      spaced by a few thousand clocks of other work: K row by row between the conversions here (a row's registers are
        //      free once it is converted), Q after the barrier below, V after the diagonal inverse.  Issued in one burst, the
        //      workgroup's 56 load instructions queue in the compute unit's memory pipeline (about 16 clocks each, behind the
        //      other workgroup's and the output stores) and every wave stands in the issue for one to two thousand clocks.
        char* const Kt_ = (GV == 2 && hsel == 1) ? Qt : Kt;     // where the group's shared tensor goes
        GDN_FETCH_DESCRIPTORS(nxt);
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int i = ROWS * tg + r;
            const int off = i * RBY + (((d0 >> 3) ^ swz<D>(i)) << 4);
            float kv[8], qv[8], vv[8];
            EL::unpack(kraw[r], kv);
            if (GV == 1) EL::unpack(qraw[r], qv);
            EL::unpack(vraw[r], vv);
            half8 kh, qh, vh;
#pragma unroll
            for (int e = 0; e < 8; ++e) { kh[e] = (half_t)kv[e]; vh[e] = (half_t)vv[e]; }
            *reinterpret_cast<half8*>(Kt_ + off) = kh;
            if (GV == 1) {
#pragma unroll
                for (int e = 0; e < 8; ++e) qh[e] = (half_t)qv[e];
                *reinterpret_cast<half8*>(Qt + off) = qh;
            }
            *reinterpret_cast<half8*>(Vt + off) = vh;
            __builtin_amdgcn_sched_barrier(0);
            GDN_FETCH_K(r, tg, d0);
            __builtin_amdgcn_sched_barrier(0);
        }
        GDN_PHASE(1);
        GDN_FETCH_GATES(nxt, lane);
        GDN_PHASE(2);
        __syncthreads();
        GDN_PHASE(3);

        // operand over d_k columns 32 s + 8 g4 .. + 7 of row 16 blk + m of a tile
        GDN_FETCH_ALL(GDN_FETCH_Q, tg, d0);
        auto row_frag = [&](const char* tile, int blk, int s) -> half8 {
            return *reinterpret_cast<const half8*>(tile + row_b[s] + blk * 16 * RBY);
        };

        // ---- preparation.  Wave a: block row a of L (diagonal inverse T_aa, the blocks -T_aa L_ac, T_aa diag(b),
        //      -T_aa diag(b gam)) and the P blocks of query block ia = 3 - a.
        {
            const int ab = wave, ia = 3 - wave;
            half8 ka[SS], qf[SS];      // K rows of block ab and Q rows of block ia as operands over d_k
#pragma unroll
            for (int s = 0; s < SS; ++s) {
                ka[s] = row_frag(Kt, ab, s);
                qf[s] = row_frag(Qt, ia, s);
            }
            // diagonal block: raw gram (symmetric), scaled into the tiles of D and of D^T
            f32x4 gr = {0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < SS; ++s) gr = mma32(ka[s], ka[s], gr);
            const f32x4 gi = *reinterpret_cast<const f32x4*>(gS + 16 * ab + 4 * g4);
            const f32x4 bi = *reinterpret_cast<const f32x4*>(bS + 16 * ab + 4 * g4);
            const float gj = gS[16 * ab + m], bj = bS[16 * ab + m];
            f32x4 d, dt;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = 4 * g4 + e;
                d[e] = (m < i) ? bi[e] * EL::exp_(fminf(gi[e] - gj, 0.f)) * gr[e] : 0.f;     // D[i][m]
                dt[e] = (i < m) ? bj * EL::exp_(fminf(gj - gi[e], 0.f)) * gr[e] : 0.f;       // D[m][i]
            }
            const f32x4 y = inv16_tiles(d, dt, m, g4);
            // T_aa from the accumulator layout to its transpose through the wave's own LDS patch (a wave's LDS
            // accesses execute in order)
#pragma unroll
            for (int e = 0; e < 4; ++e) Tf[(4 * g4 + e) * SM::TF_LD + m] = y[e];
            const f32x4 at = *reinterpret_cast<const f32x4*>(Tf + m * SM::TF_LD + 4 * g4);   // T[m][4 g4 + e]
            {
                const f32x4 gm = *reinterpret_cast<const f32x4*>(gamS + 16 * ab + 4 * g4);
                f32x4 tb, tgm;
#pragma unroll
                for (int e = 0; e < 4; ++e) { tb[e] = at[e] * bi[e]; tgm[e] = -tb[e] * gm[e]; }
                *reinterpret_cast<half8*>(tbtg + (ab * 16 + m) * PLD + 8 * g4) = cat8(cvt4(tb), cvt4(tgm));
            }
            GDN_PHASE(4);
            GDN_FETCH_ALL(GDN_FETCH_V, tg, d0);
            const float gq = gS[16 * ia + m];
            // key blocks c: left of the diagonal of block row ab, L_ac -> -(T_aa L_ac) stored by rows; up to query
            // block ia, P (rows j = keys in registers, lane = query i)
            for (int c = 0; c < 4; ++c) {
                if (c >= ab && c > ia) continue;
                half8 kc[SS];
#pragma unroll
                for (int s = 0; s < SS; ++s) kc[s] = row_frag(Kt, c, s);
                if (c < ab) {
                    f32x4 acc = {0, 0, 0, 0};
#pragma unroll
                    for (int s = 0; s < SS; ++s) acc = mma32(ka[s], kc[s], acc);   // rows i in block ab, lanes j in block c
                    const float sj = sS[16 * c + m];
                    const f32x4 ri = *reinterpret_cast<const f32x4*>(rS + c * C + 16 * ab + 4 * g4);
                    f32x4 lt;
#pragma unroll
                    for (int e = 0; e < 4; ++e) lt[e] = (bi[e] * ri[e]) * (sj * acc[e]);   // L_ac[4 g4 + e][m]
                    const f32x4 zero = {0, 0, 0, 0};
                    const f32x4 mt_ = mm16_rr(zero, lt, at);     // (L^T T^T): element e of lane (m, g4) = (T L)[m][4 g4 + e]
                    f32x4 neg;
#pragma unroll
                    for (int e = 0; e < 4; ++e) neg[e] = -mt_[e];
                    *reinterpret_cast<half4*>(mimg + (SM::m_pair(ab, c) * 16 + m) * PLD + 8 * g4 + 4 * (c & 1)) = cvt4(neg);
                }
                if (c <= ia) {
                    f32x4 acc = {0, 0, 0, 0};
#pragma unroll
                    for (int s = 0; s < SS; ++s) acc = mma32(kc[s], qf[s], acc);
                    f32x4 p;
                    if (c < ia) {   // a block below the diagonal: every key is visible, the decay factors
                        const float pr = a.scale * rS[c * C + 16 * ia + m];
                        const f32x4 sk = *reinterpret_cast<const f32x4*>(sS + 16 * c + 4 * g4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) p[e] = pr * (sk[e] * acc[e]);
                    } else {
                        const f32x4 gk = *reinterpret_cast<const f32x4*>(gS + 16 * c + 4 * g4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float val = a.scale * EL::exp_(fminf(gq - gk[e], 0.f)) * acc[e];
                            p[e] = (4 * g4 + e <= m) ? val : 0.f;
                        }
                    }
                    *reinterpret_cast<half4*>(pimg + (SM::p_pair(ia, c) * 16 + m) * PLD + 8 * g4 + 4 * (c & 1)) = cvt4(p);
                }
            }
        }
        GDN_PHASE(5);
        __syncthreads();
        if (state_pending) {   // a chain's first chunk: its start state (and, with it, the next chunk's rows) must have landed
            wait_vmcnt<0>();
            state_pending = false;
        }

        GDN_PHASE(6);
        // ---- recurrence step of this chunk, d_v columns WC wave + 16 nt + m
        {
            half8 sf[SS][NT];        // the state as an operand over d_k: step s = state tiles 2 s, 2 s + 1
#pragma unroll
            for (int s = 0; s < SS; ++s)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) sf[s][nt] = cat8(cvt4(accS[2 * s][nt]), cvt4(accS[2 * s + 1][nt]));
            // U as an operand over the tokens of block pair p (blocks 2 p, 2 p + 1); a block not yet computed reads as zero
            half8 uh[2][NT];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int e = 0; e < 8; ++e) uh[p][nt][e] = (half_t)0.f;
            const int64_t row0 = (int64_t)l * a.T_alloc + cur.tok0;
            // the outputs of this item: rows of H_v d_v elements, this head's d_v columns; byte offsets of lane (m = token, g4)
            constexpr int OB = O_BF16 ? 2 : 4;
            const int o_step = a.H_v * DV * OB;
            const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(
                reinterpret_cast<char*>(a.o) + ((row0 * a.H_v + hv) * DV) * OB, 0, (n - 1) * o_step + DV * OB, 0x00020000);
            const int o_lane = m * o_step + (WC * wave + 4 * g4) * OB;
            // K_a S0^T (tokens in registers) and (Q_a S0^T)^T (d_v in registers, lane = token) of block row ab: 16 independent
            // products.  They are issued one block row ahead, in between the short dependent products of the substitution.
            auto state_products = [&](int ab, f32x4 (&ks)[NT], f32x4 (&ot)[NT]) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) { ks[nt] = f32x4{0, 0, 0, 0}; ot[nt] = f32x4{0, 0, 0, 0}; }
#pragma unroll
                for (int s = 0; s < SS; ++s) {
                    const half8 kfr = row_frag(Kt, ab, s);
                    const half8 qfr = row_frag(Qt, ab, s);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        ks[nt] = mma32(kfr, sf[s][nt], ks[nt]);
                        ot[nt] = mma32(sf[s][nt], qfr, ot[nt]);
                    }
                }
            };
            f32x4 ks_n[NT], ot_n[NT];
            state_products(0, ks_n, ot_n);
            half8 ud[2][NT];   // diag(dec) U, like uh
#pragma unroll
            for (int ab = 0; ab < 4; ++ab) {
                const int row = 16 * ab + m;
                f32x4 ks[NT], ot[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) { ks[nt] = ks_n[nt]; ot[nt] = ot_n[nt]; }
                if (ab < 3) state_products(ab + 1, ks_n, ot_n);
                // U_a = [T_aa diag(b) | -T_aa diag(b gam)] [V_a ; K_a S0^T] + sum_c (-T_aa L_ac) U_c, two blocks c per product
                const half8 tf = *reinterpret_cast<const half8*>(tbtg + (ab * 16 + m) * PLD + 8 * g4);
                f32x4 u[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const half4 vt = tr_read(Vt + tv[nt] + ab * 16 * RBY);
                    const f32x4 zero = {0, 0, 0, 0};
                    u[nt] = mma32(tf, cat8(vt, cvt4(ks[nt])), zero);
                }
#pragma unroll
                for (int p = 0; p < 2; ++p)
                    if (2 * p < ab) {
                        const half8 mf = *reinterpret_cast<const half8*>(mimg + (SM::m_pair(ab, 2 * p) * 16 + m) * PLD + 8 * g4);
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) u[nt] = mma32(mf, uh[p][nt], u[nt]);
                    }
                const f32x4 dc = *reinterpret_cast<const f32x4*>(decS + 16 * ab + 4 * g4);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const half4 h = cvt4(u[nt]);
                    f32x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = u[nt][e] * dc[e];
                    const half4 hd = cvt4(x);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        uh[ab >> 1][nt][4 * (ab & 1) + e] = h[e];
                        ud[ab >> 1][nt][4 * (ab & 1) + e] = hd[e];
                    }
                }
                // O_a^T = diag(gam scale) (Q_a S0^T)^T + sum_{c <= a} U_c^T P_ac^T   (lane = token)
                const float gm = gamS[row] * a.scale;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) ot[nt][e] *= gm;
#pragma unroll
                for (int p = 0; p < 2; ++p)
                    if (2 * p <= ab) {
                        const half8 pf = *reinterpret_cast<const half8*>(pimg + (SM::p_pair(ab, 2 * p) * 16 + m) * PLD + 8 * g4);
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) ot[nt] = mma32(uh[p][nt], pf, ot[nt]);
                    }
                // The next item's inputs (fetched at staging time) must have landed before this item's first store is
                // issued: loads and stores share one in-flight counter, and with both kinds pending the first use of a
                // fetched register would wait for every store to be acknowledged (thousands of cycles at the top of the
                // next item).  Here the fetch is thousands of cycles old and nothing else is pending, so this costs nothing.
                if (ab == 0) {
                    wait_vmcnt<0>();
                    if (draw_pending) {     // the draw made at the top of this item has returned with the loads
                        if (wave == 0 && hsel == 0 && lane_ == 0) reserve_lds[0] = drawn;
                        draw_pending = false;
                    }
                }
                // buffer stores through the item's output descriptor (it ends with the chunk's last row: rows past n are dropped)
                if (O_BF16) {
                    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)   // v_cvt_pk_bf16_f32: round to nearest even, two values per instruction
                        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, __builtin_convertvector(ot[nt], bf16x4)), ro,
                                                              o_lane + ab * 16 * o_step + 32 * nt, 0, 0);
                } else {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, ot[nt]), ro, o_lane + ab * 16 * o_step + 64 * nt, 0, 0);
                }
            }
            GDN_PHASE(7);
            // state update: S^T = gam_C S^T + sum_j K^T[.][j] (dec_j U[j][.]), two token blocks per product
            const float gam_last = gamS[C - 1];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const char* kt = Kt + tr_b[mt >> 1] + 8 * (mt & 1);
                const half8 k0 = cat8(tr_read(kt), tr_read(kt + 16 * RBY));
                const half8 k1 = cat8(tr_read(kt + 32 * RBY), tr_read(kt + 48 * RBY));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) accS[mt][nt][e] *= gam_last;
                    accS[mt][nt] = mma32(k0, ud[0][nt], accS[mt][nt]);
                    accS[mt][nt] = mma32(k1, ud[1][nt], accS[mt][nt]);
                }
            }
            GDN_PHASE(8);
            // checkpoint emission: exact state after the last token of this chunk
            const int eslot = cur.eslot;   // looked up one item ahead, with the chunk's other bookkeeping
            if (eslot >= 0) {
                float* dst = a.state_dst + eslot * a.dst_slot_stride + head_off;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        *reinterpret_cast<f32x4*>(dst + (WC * wave + 16 * nt + m) * DK + 32 * (mt >> 1) + 8 * g4 + 4 * (mt & 1)) = accS[mt][nt];
            }
        }

        GDN_PHASE(9);
        if (nxt.chain < 0) break;
        cur = nxt;
    }
}

#undef GDN_FETCH_DESCRIPTORS
#undef GDN_FETCH_ALL
#undef GDN_FETCH_K
#undef GDN_FETCH_Q
#undef GDN_FETCH_V
#undef GDN_FETCH_GATES

}  // namespace gdn
