// Device side of the attention layers' part of a cache hit (see include/attn_resume.h): the
// append of the suffix's keys and values to the cache, and causal softmax attention of the suffix
// over positions 1 .. its own, for gfx950 (wave64, bf16 matrix cores, fp32 accumulation).
//
// Attention kernel.  One workgroup of four waves owns ATT_BQ = 128 consecutive suffix tokens of
// one (request, query head); wave w owns 32 of them, one per lane column.  Key/value rows are
// walked in tiles of 64 (32 at d = 256), each tile brought into one of two LDS stages by 16-byte
// buffer loads to LDS (no registers) while the waves compute on the other stage.
//
// Both contractions are computed transposed, so that a query is a COLUMN of every accumulator
// tile and everything a softmax row needs sits in one lane (and its partner 32 lanes up):
//   S^T[kv][q] = sum_d K[kv][d] Q[q][d]      A = a key tile row (16-byte LDS read), B = the
//                                            query fragment, held in registers for the whole walk
//   O^T[dv][q] += sum_kv V^T[dv][kv] P^T[kv][q]
//                                            (fp16 operands: the value cache is kept in fp16)
//                                            B = the weights, packed to fp16 straight from the
//                                            S^T accumulators: accumulator register 4b+e of
//                                            half-wave g holds row 8b+4g+e, so registers 8s..8s+7
//                                            are rows 16s+4g+{0..3} and 16s+8+4g+{0..3}; A = the
//                                            same two runs of four kv rows of one value column,
//                                            which is what the 16-bit LDS transpose read returns
//                                            (lane i of a group of 16 receives element i%4 of the
//                                            8-byte rows addressed by lanes i/4, i/4+4, i/4+8,
//                                            i/4+12 of the group).
// Calls whose suffixes are short against the 128 rows of a workgroup pack the query heads of a key/value group
// into the rows instead (row = token * G + head of the group, 128 / G tokens per workgroup): the rows of a
// workgroup then all share one key/value head anyway, and a 16-token suffix fills the rows that 16 tokens of one
// head would leave empty.  Nothing else changes: a row's arithmetic does not depend on which lane carries it.
//
// A call with too few (request, head, 128-token) pieces to fill the chip splits the key walk of a
// piece into parts of whole tiles: each part is a workgroup that leaves its unnormalised O, running
// maximum and normaliser in a workspace slot, and a second kernel merges the parts of a piece.
//
// LDS rows are unpadded (a load to LDS writes a wave's 64 x 16 bytes contiguously); bank
// conflicts are avoided by storing 16-byte chunk c of row r at chunk position c ^ f(r), with f
// chosen per tile for its read pattern (16 rows x same chunk for keys, 4 rows x 4 chunks for values).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2 __attribute__((ext_vector_type(2)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int ATT_BQ = 128;       // rows (query columns of the accumulators) per workgroup
// key/value rows per tile (a multiple of 32): 64, and 32 at d = 256, where the shorter tile brings the
// kernel under 256 registers and two workgroups onto a compute unit
__host__ __device__ constexpr int att_kt(int d) { return d == 256 ? 32 : 64; }
constexpr int ATT_THREADS = 256;
constexpr int APPEND_THREADS = 256;

struct AttnArgs {
    const uint16_t* q;        // [T][H_q][D]
    const uint16_t* gate;     // [T][H_q][D] or nullptr
    const uint16_t* k_cache;  // slots of [cap][H_kv][D]
    const uint16_t* v_cache;  // fp16 bits
    void* o;                  // [T][H_q][D], float or bf16
    const int32_t* cu;        // device: n_req + 1
    const int32_t* start;     // device: n_req
    const int32_t* slot;      // device: n_req
    const int32_t* unit_req;  // device: n_units, heaviest first
    const int32_t* unit_tile; // device: index of the 128-token tile inside the request
    const int32_t* unit_t0;   // device: first key tile of the unit
    const int32_t* unit_t1;   // device: one past its last key tile
    const int32_t* unit_part; // device: workspace slot of a partial result, or -1: the unit is a whole walk
    float* part_o;            // [slot][H_q][ATT_BQ][D] unnormalised partial outputs
    float* part_ml;           // [slot][H_q][ATT_BQ][2] running maximum (raw logits) and normaliser
    int64_t slot_stride;      // elements
    int32_t n_units;
    int32_t H_q, H_kv;
    int32_t xcd_split;        // 1: blocks are dealt to the 8 XCDs by key/value head
    int32_t pack;             // query heads per token in a workgroup's rows: 1, or H_q / H_kv (a divisor of 128)
    float scale_log2e;        // scale * log2(e)
};

struct AppendArgs {
    const uint16_t* k_new;    // [T][H_kv][D]
    const uint16_t* v_new;
    uint16_t* k_cache;
    uint16_t* v_cache;        // fp16 bits
    const int32_t* cu;
    const int32_t* start;
    const int32_t* slot;
    int64_t slot_stride;
    int64_t n_chunks;         // T * row_chunks
    int32_t n_req;
    int32_t row_chunks;       // 16-byte chunks per token row: H_kv * D / 8
};

// s_waitcnt vmcnt(N) (gfx9 encoding: vmcnt in bits 3:0 and 15:14; other counters left alone)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(((N & 0x30) << 10) | (N & 0xF) | 0x0F70);
}

// One wave-wide 16-byte-per-lane buffer load to LDS: lane i's chunk lands at lds + 16 i.  The descriptor covers
// `bytes` from `base`; a lane whose byte offset voff + soff lies past it writes zeros.
__device__ __forceinline__ void load_to_lds(const void* base, int bytes, char* lds, int voff, int soff) {
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)lds, 16, voff, soff, 0, 0);
}

// max / sum of a value with the lane 32 up or down (one swap instruction, no LDS)
__device__ __forceinline__ float max_with_other_half(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto p = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (unsigned)p[0]), __builtin_bit_cast(float, (unsigned)p[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto p = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (unsigned)p[0]) + __builtin_bit_cast(float, (unsigned)p[1]);
}

// Appends the suffix's key and value rows to the cache rows start .. start+n-1 of each request's
// slot: one 16-byte chunk of k and of v per thread, the values widened from bf16 to fp16.
__global__ void __launch_bounds__(APPEND_THREADS) attn_append_kernel(AppendArgs a) {
    const int64_t id = (int64_t)blockIdx.x * APPEND_THREADS + threadIdx.x;
    if (id >= a.n_chunks) return;
    const int32_t t = (int32_t)(id / a.row_chunks);
    const int32_t c = (int32_t)(id - (int64_t)t * a.row_chunks);
    int lo = 0, hi = a.n_req;                       // request with cu[r] <= t < cu[r+1]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.cu[mid] <= t) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int64_t row = (int64_t)a.start[r] + (t - a.cu[r]);
    const int64_t dst = (int64_t)a.slot[r] * a.slot_stride + (row * a.row_chunks + c) * 8;
    const int64_t src = ((int64_t)t * a.row_chunks + c) * 8;
    *reinterpret_cast<u32x4*>(a.k_cache + dst) = *reinterpret_cast<const u32x4*>(a.k_new + src);
    const u32x4 vb = *reinterpret_cast<const u32x4*>(a.v_new + src);
    half8 vh;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        vh[2 * i] = (_Float16)__builtin_bit_cast(float, vb[i] << 16);
        vh[2 * i + 1] = (_Float16)__builtin_bit_cast(float, vb[i] & 0xffff0000u);
    }
    *reinterpret_cast<u32x4*>(a.v_cache + dst) = __builtin_bit_cast(u32x4, vh);
}

template <int D>
struct AttnSmem {
    static constexpr int CPR = D / 8;                     // 16-byte chunks per row
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int KT = att_kt(D);                  // key/value rows per tile
    static constexpr int TILE_BYTES = KT * ROW_BYTES;
    static constexpr int K_OFF = 0, V_OFF = TILE_BYTES;
    static constexpr int STAGE_BYTES = 2 * TILE_BYTES;
    static constexpr int BYTES = 2 * STAGE_BYTES;
    static constexpr int PIECES = TILE_BYTES / 1024;      // 1 KiB wave-wide loads per tile
    static_assert(D == 64 || D == 128 || D == 256, "head size");
    static_assert(PIECES % 4 == 0, "pieces split evenly over four waves");
    // chunk position swizzles
    static __device__ __forceinline__ int fk(int row) { return CPR >= 16 ? (row & 15) : ((row >> 1) & 7); }
    static __device__ __forceinline__ int fv(int row) { return CPR >= 16 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};

template <int D, typename OT>
__global__ void __launch_bounds__(ATT_THREADS, 2) attn_suffix_kernel(AttnArgs a) {
    typedef AttnSmem<D> SM;
    constexpr int CPR = SM::CPR;
    constexpr int KB = D / 16;      // contraction steps of S^T
    constexpr int RB = D / 32;      // row tiles of O^T
    constexpr int ATT_KT = SM::KT;
    constexpr int ATT_KVB = ATT_KT / 32;   // 32-row accumulator tiles of S^T per key tile
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31;      // query column of this lane
    const int g = lane >> 5;        // half-wave

    // ---- which (unit, head block): a head block is one query head, or with packed rows the heads of one group
    const int R = a.pack;                 // query heads per token in this workgroup's rows
    const int per = a.H_q / a.H_kv / R;   // head blocks per key/value head: the group size, or 1
    int item, hb;
    if (a.xcd_split) {
        const int X = 8 / a.H_kv;                 // XCDs per key/value head
        const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3;
        const int sub = xcd / a.H_kv;
        const int64_t e = (int64_t)k * X + sub;
        if (e >= (int64_t)a.n_units * per) return;
        item = (int)(e / per);
        hb = (xcd % a.H_kv) * per + (int)(e % per);
    } else {
        const int HB = a.H_q / R;
        item = blockIdx.x / HB;
        hb = blockIdx.x % HB;
    }
    const int kvh = hb / per;
    const int TPW = ATT_BQ / R;           // tokens per workgroup
    const int wrow = 32 * wave + col;     // this lane's row of the workgroup: token wrow / R, head hb * R + wrow % R
    const int tl = wrow / R;
    const int hq = hb * R + (wrow - tl * R);
    const int r = a.unit_req[item];
    const int q0 = a.unit_tile[item] * TPW;
    const int t0 = a.unit_t0[item], t1 = a.unit_t1[item];  // key tiles [t0, t1) of this unit
    const int part = a.unit_part[item];
    const int tok0 = a.cu[r];
    const int n = a.cu[r + 1] - tok0;
    const int c0 = a.start[r];
    const int q_end = min(q0 + TPW, n);                    // suffix tokens of this workgroup: [q0, q_end)
    const int kv_len = c0 + q_end;                         // key rows any of them may see
    const int wq0 = q0 + (32 * wave) / R;                  // first token of this wave
    const int wq1 = min(q0 + (32 * wave + 31) / R + 1, q_end);   // one past its last
    const int n_tiles_w = wq0 < q_end ? (c0 + wq1 + ATT_KT - 1) / ATT_KT : 0;   // tiles this wave can see
    const bool valid = q0 + tl < q_end;                    // this lane's row is a token of the request
    const int qrow = min(q0 + tl, q_end - 1);              // clamped: lanes past the end repeat the last token
    const int lim = c0 + qrow;                             // last visible key row (0-based) of this lane's query

    // ---- tile loader: wave w brings pieces [w*PPW, (w+1)*PPW) of the key and of the value tile, one 16-byte
    // chunk per lane and piece, by buffer loads to LDS.  The descriptors cover rows [0, kv_len) of the request's
    // slot: lanes of rows past kv_len (the ragged end of the last tile) write zeros, which the mask never weighs.
    // A lane's offset inside a piece does not change from tile to tile; the tile and piece move in the scalar offset.
    constexpr int PPW = SM::PIECES / 4;                    // pieces per wave and tensor
    constexpr int RPP = 64 / CPR;                          // rows per piece
    const int row_bytes = a.H_kv * D * 2;
    const uint16_t* const kslot = a.k_cache + (int64_t)a.slot[r] * a.slot_stride;
    const uint16_t* const vslot = a.v_cache + (int64_t)a.slot[r] * a.slot_stride;
    const int slot_bytes = kv_len * row_bytes;
    int koff[PPW], voff[PPW];
#pragma unroll
    for (int i = 0; i < PPW; ++i) {
        const int s = (wave * PPW + i) * 64 + lane;        // 16-byte slot inside the tile
        const int row = s / CPR, pos = s % CPR;
        const int in_piece = (row - (wave * PPW + i) * RPP) * row_bytes + kvh * D * 2;
        koff[i] = in_piece + ((pos ^ SM::fk(row)) << 4);
        voff[i] = in_piece + ((pos ^ SM::fv(row)) << 4);
    }
    auto issue = [&](int t, int stage) {
        char* const sb = smem + stage * SM::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < PPW; ++i) {
            const int p = wave * PPW + i;
            const int soff = (t * ATT_KT + p * RPP) * row_bytes;
            load_to_lds(kslot, slot_bytes, sb + SM::K_OFF + p * 1024, koff[i], soff);
            load_to_lds(vslot, slot_bytes, sb + SM::V_OFF + p * 1024, voff[i], soff);
        }
    };
    issue(t0, 0);

    // ---- query fragments: B operand of S^T, d = 16*kb + 8*g + {0..7}
    bf16x8 qf[KB];
    {
        const uint16_t* const qp = a.q + ((int64_t)(tok0 + qrow) * a.H_q + hq) * D + 8 * g;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) qf[kb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + 16 * kb));
    }

    f32x16 O[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[rb][i] = 0.f;
    float m = -INFINITY;     // running maximum of the raw logits of this lane's query (both half-waves agree)
    float l = 0.f;           // this half-wave's share of the normaliser
    const float c = a.scale_log2e;

    // per-lane LDS byte offsets inside a stage
    const int krow_off = col * SM::ROW_BYTES;                       // + 32*kvblk rows
    const int kz = g ^ SM::fk(col);                                 // chunk position of step kb: (2*kb) ^ kz
    const int i16 = lane & 15, b4 = (lane >> 4) & 1;
    const int vrow = 4 * g + (i16 >> 2);                            // + 16*s + 8*grp rows
    const int vfv = SM::fv(vrow);
    const int vrow_off = SM::V_OFF + vrow * SM::ROW_BYTES + 8 * (i16 & 1);
    const int vchunk = 2 * b4 + ((i16 & 3) >> 1);                   // + 4*rb

    for (int t = t0; t < t1; ++t) {
        const int stage = (t - t0) & 1;
        wait_vmcnt<0>();
        __syncthreads();                       // tile t has landed; everyone has left the other stage
        if (t >= n_tiles_w) {                  // wave-uniform: nothing of this tile is visible to this wave
            issue(t + 1, stage ^ 1);
            continue;
        }
        const char* const sb = smem + stage * SM::STAGE_BYTES;
        const int kv0 = t * ATT_KT;
        // The next tile's loads are issued in between the matrix instructions of S^T (issuing one takes some
        // tens of cycles, which a matrix instruction in flight covers).  Past the unit's last tile the loads
        // are issued all the same: they stay inside the slot, or are cut to zeros by the descriptor, and land
        // in the stage nobody reads.
        issue(t + 1, stage ^ 1);

        // ---- S^T = K Q^T, in 32-row tiles
        f32x16 S[ATT_KVB];
#pragma unroll
        for (int kvb = 0; kvb < ATT_KVB; ++kvb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) S[kvb][i] = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const bf16x8 kf = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const u32x4*>(sb + SM::K_OFF + kvb * 32 * SM::ROW_BYTES + krow_off + (((2 * kb) ^ kz) << 4)));
                S[kvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kb], S[kvb], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);            // four key fragments ahead
#pragma unroll
        for (int i = 0; i < ATT_KVB * KB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);        // one key fragment read
            if (i < 2 * PPW) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one load to LDS
        }
        // ---- causal mask on the tiles that reach past the first row's limit
        if (kv0 + ATT_KT - 1 > c0 + wq0) {
#pragma unroll
            for (int kvb = 0; kvb < ATT_KVB; ++kvb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int kv = kv0 + 32 * kvb + 8 * (i >> 2) + 4 * g + (i & 3);
                    if (kv > lim) S[kvb][i] = -INFINITY;
                }
        }
        // ---- online softmax for this lane's query
        float mx = S[0][0];
#pragma unroll
        for (int kvb = 0; kvb < ATT_KVB; ++kvb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[kvb][i]);
        mx = max_with_other_half(mx);
        const float m_new = fmaxf(m, mx);
        // -inf only in a part of a split walk whose first tiles lie past this query's limit: nothing to weigh yet
        const float m_ref = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m - m_ref) * c);
        const float mc = m_ref * c;
        m = m_new;
        half8 pf[2 * ATT_KVB];                 // B operands of the 16-row steps
        float lsum = 0.f;
#pragma unroll
        for (int s = 0; s < 2 * ATT_KVB; ++s) {
            f32x2 e[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                e[j][0] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[s >> 1][8 * (s & 1) + 2 * j], c, -mc));
                e[j][1] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[s >> 1][8 * (s & 1) + 2 * j + 1], c, -mc));
            }
            half2 h[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                h[j] = __builtin_convertvector(e[j], half2);
                const half2 one = {(_Float16)1.0f, (_Float16)1.0f};
                lsum = __builtin_amdgcn_fdot2(h[j], one, lsum, false);   // the sum of the ROUNDED weights
            }
            pf[s] = __builtin_shufflevector(__builtin_shufflevector(h[0], h[1], 0, 1, 2, 3),
                                            __builtin_shufflevector(h[2], h[3], 0, 1, 2, 3), 0, 1, 2, 3, 4, 5, 6, 7);
        }
        l = l * alpha + lsum;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int i = 0; i < 16; ++i) O[rb][i] *= alpha;
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int vpos = ((4 * rb + vchunk) ^ vfv) << 4;
#pragma unroll
            for (int s = 0; s < 2 * ATT_KVB; ++s) {
                const char* const p0 = sb + vrow_off + vpos + (16 * s) * SM::ROW_BYTES;
                const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p0));
                const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p0 + 8 * SM::ROW_BYTES));
                const half8 vf = __builtin_bit_cast(half8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                O[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[s], O[rb], 0, 0, 0);
            }
        }
    }

    wait_vmcnt<0>();                           // no load to LDS may be in flight when the workgroup's LDS is given back
    // ---- a part of a split walk leaves its unnormalised result in its workspace slot
    if (part >= 0) {
        if (valid) {
            const int64_t prow = ((int64_t)part * (a.H_q / R) + hb) * ATT_BQ + wrow;
            const float lt = sum_with_other_half(l);
            if (g == 0) *reinterpret_cast<f32x2*>(a.part_ml + prow * 2) = f32x2{m, lt};
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    *reinterpret_cast<f32x4*>(a.part_o + prow * D + 32 * rb + 8 * b + 4 * g) =
                        f32x4{O[rb][4 * b], O[rb][4 * b + 1], O[rb][4 * b + 2], O[rb][4 * b + 3]};
        }
        return;
    }
    // ---- normalise, gate, store: register 4b+e of tile rb is value column 32*rb + 8*b + 4*g + e
    if (valid) {
        const float inv = 1.f / sum_with_other_half(l);
        const int64_t base = ((int64_t)(tok0 + q0 + tl) * a.H_q + hq) * D;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int dv = 32 * rb + 8 * b + 4 * g;
                f32x4 y = {O[rb][4 * b] * inv, O[rb][4 * b + 1] * inv, O[rb][4 * b + 2] * inv, O[rb][4 * b + 3] * inv};
                if (a.gate) {
                    const u32x2 gb = *reinterpret_cast<const u32x2*>(a.gate + base + dv);
                    const float g0 = __builtin_bit_cast(float, gb[0] << 16), g1 = __builtin_bit_cast(float, gb[0] & 0xffff0000u);
                    const float g2 = __builtin_bit_cast(float, gb[1] << 16), g3 = __builtin_bit_cast(float, gb[1] & 0xffff0000u);
                    y[0] *= 1.f / (1.f + __expf(-g0));
                    y[1] *= 1.f / (1.f + __expf(-g1));
                    y[2] *= 1.f / (1.f + __expf(-g2));
                    y[3] *= 1.f / (1.f + __expf(-g3));
                }
                if constexpr (sizeof(OT) == 4) {
                    *reinterpret_cast<f32x4*>(static_cast<float*>(a.o) + base + dv) = y;
                } else {
                    const bf16x4 yb = __builtin_convertvector(y, bf16x4);
                    *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.o) + base + dv) = __builtin_bit_cast(u32x2, yb);
                }
            }
    }
}

struct CombineArgs {
    const float* part_o;
    const float* part_ml;
    const uint16_t* gate;     // or nullptr
    void* o;
    const int32_t* cu;
    const int32_t* piece_req;   // device: n_pieces split pieces
    const int32_t* piece_tile;
    const int32_t* piece_base;  // first workspace slot of the piece
    const int32_t* piece_parts; // its number of parts (consecutive slots)
    int32_t H_q;
    int32_t pack;               // as in AttnArgs
    float scale_log2e;
};

// Merges the parts of one split piece for one query head: o = sum_p w_p O_p / sum_p w_p l_p with
// w_p = 2^((m_p - max_p m_p) * scale * log2 e); a part that saw no key has m_p = -inf, weight 0 and O_p = 0.
// One thread per (row, four value columns), COMBINE_SUBS workgroups per (piece, head); the loads of all
// parts are independent of each other, so the pass costs a few memory round trips, not one per part.
template <int D>
struct CombineShape {
    static constexpr int CH = D / 4;                               // threads per row
    static constexpr int SUBS = ATT_BQ * CH / ATT_THREADS;         // workgroups per (piece, head)
};

template <int D, typename OT>
__global__ void __launch_bounds__(ATT_THREADS) attn_combine_kernel(CombineArgs a) {
    constexpr int CH = CombineShape<D>::CH, SUBS = CombineShape<D>::SUBS;
    const int ph = blockIdx.x / SUBS, sub = blockIdx.x % SUBS;
    const int R = a.pack, HB = a.H_q / R, TPW = ATT_BQ / R;
    const int piece = ph / HB, hb = ph % HB;
    const int r = a.piece_req[piece];
    const int q0 = a.piece_tile[piece] * TPW;
    const int tok0 = a.cu[r];
    const int rows = min(TPW, a.cu[r + 1] - tok0 - q0) * R;
    const int base = a.piece_base[piece], P = a.piece_parts[piece];
    {
        const int idx = sub * ATT_THREADS + threadIdx.x;
        const int row = idx / CH, ch = idx - row * CH;
        if (row >= rows) return;
        const int64_t prow0 = ((int64_t)base * HB + hb) * ATT_BQ + row;
        const int64_t pstep = (int64_t)HB * ATT_BQ;                   // rows between consecutive parts
        const int tl = row / R, hq = hb * R + (row - tl * R);
        float M = -INFINITY;
#pragma unroll 4
        for (int p = 0; p < P; ++p) M = fmaxf(M, a.part_ml[(prow0 + p * pstep) * 2]);   // finite: part 0 sees key row 0
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float L = 0.f;
#pragma unroll 4
        for (int p = 0; p < P; ++p) {
            const int64_t prow = prow0 + p * pstep;
            const f32x2 ml = *reinterpret_cast<const f32x2*>(a.part_ml + prow * 2);
            const f32x4 op = *reinterpret_cast<const f32x4*>(a.part_o + prow * D + 4 * ch);
            const float w = __builtin_amdgcn_exp2f((ml[0] - M) * a.scale_log2e);
            acc[0] += w * op[0]; acc[1] += w * op[1]; acc[2] += w * op[2]; acc[3] += w * op[3];
            L += w * ml[1];
        }
        const float inv = 1.f / L;
        f32x4 y = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
        const int64_t at = ((int64_t)(tok0 + q0 + tl) * a.H_q + hq) * D + 4 * ch;
        if (a.gate) {
            const u32x2 gb = *reinterpret_cast<const u32x2*>(a.gate + at);
            const float g0 = __builtin_bit_cast(float, gb[0] << 16), g1 = __builtin_bit_cast(float, gb[0] & 0xffff0000u);
            const float g2 = __builtin_bit_cast(float, gb[1] << 16), g3 = __builtin_bit_cast(float, gb[1] & 0xffff0000u);
            y[0] *= 1.f / (1.f + __expf(-g0));
            y[1] *= 1.f / (1.f + __expf(-g1));
            y[2] *= 1.f / (1.f + __expf(-g2));
            y[3] *= 1.f / (1.f + __expf(-g3));
        }
        if constexpr (sizeof(OT) == 4) {
            *reinterpret_cast<f32x4*>(static_cast<float*>(a.o) + at) = y;
        } else {
            const bf16x4 yb = __builtin_convertvector(y, bf16x4);
            *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.o) + at) = __builtin_bit_cast(u32x2, yb);
        }
    }
}

}  // namespace attn
