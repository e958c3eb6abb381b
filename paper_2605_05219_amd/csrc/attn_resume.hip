// attn_resume: host side of the attention layers' part of a cache hit (see include/attn_resume.h).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "attn_kernel.h"
#include "attn_resume.h"
#include "gdn_host.h"

namespace attn {
namespace {

inline int32_t hip_err(hipError_t e) { return e == hipSuccess ? GDN_OK : GDN_ERR_HIP - (int32_t)e; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int32_t check_shape(const attn_shape* s) {
    if (!s) return GDN_ERR_NULL;
    if (s->H_q <= 0 || s->H_kv <= 0 || s->H_q % s->H_kv != 0) return GDN_ERR_SHAPE;
    if (s->d != 64 && s->d != 128 && s->d != 256) return GDN_ERR_SHAPE;
    if (s->o_dtype != GDN_F32 && s->o_dtype != GDN_BF16) return GDN_ERR_SHAPE;
    if (!(s->scale > 0.f) || !std::isfinite(s->scale)) return GDN_ERR_SHAPE;
    return GDN_OK;
}

// geometry of a pool of sequence slots
int32_t check_pool(const attn_shape* s, int64_t slot_stride, int32_t n_slots, int32_t cap) {
    if (n_slots < 0 || cap < 0) return GDN_ERR_COUNT;
    if (slot_stride < 0 || slot_stride % 8 != 0) return GDN_ERR_ALIGN;
    if (slot_stride < (int64_t)cap * s->H_kv * s->d) return GDN_ERR_SHAPE;   // slots would overlap
    // a slot is addressed with 32-bit byte offsets, which may run up to two key tiles past its last row
    if (((int64_t)cap + 128) * s->H_kv * s->d * 2 > INT32_MAX) return GDN_ERR_SHAPE;
    return GDN_OK;
}

int32_t check_slots(const int32_t* ids, int32_t n, int32_t n_slots, bool skip_empty, const int32_t* len) {
    std::vector<int32_t> seen;
    seen.reserve(n);
    for (int32_t r = 0; r < n; ++r) {
        if (ids[r] < 0 || ids[r] >= n_slots) return GDN_ERR_SLOT_RANGE;
        if (skip_empty && len[r] == 0) continue;
        seen.push_back(ids[r]);
    }
    std::sort(seen.begin(), seen.end());
    if (std::adjacent_find(seen.begin(), seen.end()) != seen.end()) return GDN_ERR_SLOT_DUP;
    return GDN_OK;
}

// Splitting the key walk: calls with fewer than SPLIT_BELOW workgroups cut the walks of their pieces
// into parts of at least SPLIT_MIN_KEYS keys (whole tiles), aiming at SPLIT_BELOW workgroups in all; the
// partial results of at most SPLIT_MAX_WGS (part, head) pairs live in the workspace.
constexpr int SPLIT_BELOW = 512;       // two workgroups per compute unit
constexpr int SPLIT_MIN_KEYS = 512;
constexpr int SPLIT_MAX_WGS = 768;

// ints of the uploaded index arrays: cu (n_req+1), start, slot (n_req each), five per unit, four per split piece
// (with packed rows a piece is 128 / G tokens, G the heads per key/value head: at most G times as many pieces)
inline int64_t max_items(int32_t n_req, int64_t T, int G) { return T * G / ATT_BQ + n_req; }
inline int64_t max_units(int32_t n_req, int64_t T, int G) { return max_items(n_req, T, G) + SPLIT_MAX_WGS; }
inline int64_t plan_ints(int32_t n_req, int64_t T, int G) {
    return 3 * (int64_t)n_req + 1 + 5 * max_units(n_req, T, G) + 4 * max_items(n_req, T, G);
}
inline int64_t plan_bytes(int32_t n_req, int64_t T, int G) {
    return (plan_ints(n_req, T, G) * (int64_t)sizeof(int32_t) + 255) / 256 * 256;
}
inline int64_t part_ml_bytes() { return (int64_t)SPLIT_MAX_WGS * ATT_BQ * 2 * sizeof(float); }
inline int64_t part_o_bytes(int d) { return (int64_t)SPLIT_MAX_WGS * ATT_BQ * d * sizeof(float); }

template <int D, typename OT>
hipError_t launch_attn(const AttnArgs& a, unsigned blocks, hipStream_t stream) {
    constexpr int smem = AttnSmem<D>::BYTES;
    // once per process, also when several host threads make their first call together
    static std::once_flag once;
    static hipError_t once_err = hipSuccess;
    std::call_once(once, [] { once_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_suffix_kernel<D, OT>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, smem); });
    if (once_err != hipSuccess) return once_err;
    hipLaunchKernelGGL((attn_suffix_kernel<D, OT>), dim3(blocks), dim3(ATT_THREADS), smem, stream, a);
    return hipGetLastError();
}

template <typename OT>
hipError_t launch_attn_d(int d, const AttnArgs& a, unsigned blocks, hipStream_t stream) {
    switch (d) {
        case 64: return launch_attn<64, OT>(a, blocks, stream);
        case 128: return launch_attn<128, OT>(a, blocks, stream);
        default: return launch_attn<256, OT>(a, blocks, stream);
    }
}

template <typename OT>
hipError_t launch_combine_d(int d, const CombineArgs& a, unsigned blocks /* (piece, head) pairs */, hipStream_t stream) {
    switch (d) {
        case 64: hipLaunchKernelGGL((attn_combine_kernel<64, OT>), dim3(blocks * CombineShape<64>::SUBS), dim3(ATT_THREADS), 0, stream, a); break;
        case 128: hipLaunchKernelGGL((attn_combine_kernel<128, OT>), dim3(blocks * CombineShape<128>::SUBS), dim3(ATT_THREADS), 0, stream, a); break;
        default: hipLaunchKernelGGL((attn_combine_kernel<256, OT>), dim3(blocks * CombineShape<256>::SUBS), dim3(ATT_THREADS), 0, stream, a); break;
    }
    return hipGetLastError();
}

// The work of one attn_suffix_prefill call (host, integer): how the rows of a workgroup are made up, the pieces
// (row tiles of a request), the cut of long key walks into parts, and the units (whole walks or parts) in launch order.
std::atomic<int32_t> g_allow_split{1}, g_allow_pack{1};   // attn_tune_split / attn_tune_pack
struct Unit { int32_t req, tile, t0, t1, part; };
struct UnitPlan {
    int pack = 1;                     // query heads per token in a workgroup's rows: 1, or H_q / H_kv
    std::vector<Unit> units;          // those with the most key tiles first
    std::vector<int32_t> piece_req, piece_tile, piece_base, piece_parts;   // the split pieces and their workspace slots
};

void build_units(const attn_shape& sh, int32_t n_req, const int32_t* len, const int32_t* start_pos, UnitPlan& out) {
    const attn_shape* s = &sh;
    // ---- rows of a workgroup: 128 tokens of one query head, or, where that would leave at least a fifth of all
    // rows empty (short suffixes), 128 / G tokens of the G heads of a key/value group
    const int KT = att_kt(s->d);
    const int G = s->H_q / s->H_kv;
    int pack = 1;
    if (G > 1 && ATT_BQ % G == 0) {
        int64_t rows_plain = 0, rows_packed = 0;
        for (int32_t r = 0; r < n_req; ++r) {
            rows_plain += (int64_t)((len[r] + ATT_BQ - 1) / ATT_BQ) * s->H_q;
            rows_packed += (int64_t)((len[r] + ATT_BQ / G - 1) / (ATT_BQ / G)) * s->H_kv;
        }
        if (rows_packed * 5 <= rows_plain * 4 && g_allow_pack.load() != 0) pack = G;
    }
    const int TPW = ATT_BQ / pack;        // tokens per workgroup
    const int HB = s->H_q / pack;         // head blocks (workgroups) per unit
    // ---- pieces: one per TPW suffix tokens of a request
    struct Piece { int32_t req, tile, n_tiles, parts; };
    std::vector<Piece> pieces;
    int64_t total_tiles = 0;
    for (int32_t r = 0; r < n_req; ++r)
        for (int32_t t = 0; t * TPW < len[r]; ++t) {
            const int32_t kv = start_pos[r] + std::min((t + 1) * TPW, len[r]);
            pieces.push_back({r, t, (kv + KT - 1) / KT, 1});
            total_tiles += pieces.back().n_tiles;
        }
    const int64_t n_items = (int64_t)pieces.size();
    // ---- too few workgroups for the chip: cut long key walks into parts
    int64_t split_wgs = 0;
    if (n_items * HB < SPLIT_BELOW && g_allow_split.load() != 0) {
        int64_t tp = std::max<int64_t>(SPLIT_MIN_KEYS / KT, (total_tiles * HB + SPLIT_BELOW - 1) / SPLIT_BELOW);
        for (;; tp *= 2) {
            split_wgs = 0;
            for (Piece& p : pieces) {
                p.parts = p.n_tiles >= 2 * tp ? (int32_t)((p.n_tiles + tp - 1) / tp) : 1;
                if (p.parts > 1) split_wgs += (int64_t)p.parts * HB;
            }
            if (split_wgs <= SPLIT_MAX_WGS) break;
        }
    }
    // ---- units: a whole walk or one part of it; those with the most key tiles first
    std::vector<Unit>& units = out.units;
    std::vector<int32_t>&piece_req = out.piece_req, &piece_tile = out.piece_tile, &piece_base = out.piece_base,
                        &piece_parts = out.piece_parts;
    int32_t next_slot = 0;
    for (const Piece& p : pieces) {
        if (p.parts == 1) {
            units.push_back({p.req, p.tile, 0, p.n_tiles, -1});
            continue;
        }
        piece_req.push_back(p.req); piece_tile.push_back(p.tile); piece_base.push_back(next_slot); piece_parts.push_back(p.parts);
        const int32_t per = (p.n_tiles + p.parts - 1) / p.parts;
        for (int32_t j = 0; j < p.parts; ++j)
            units.push_back({p.req, p.tile, j * per, std::min((j + 1) * per, p.n_tiles), next_slot++});
    }
    std::stable_sort(units.begin(), units.end(), [](const Unit& x, const Unit& y) { return x.t1 - x.t0 > y.t1 - y.t0; });
    out.pack = pack;
}

}  // namespace
}  // namespace attn

using namespace attn;

extern "C" {

int64_t attn_workspace_bytes(const attn_shape* s, int32_t n_req, int64_t total_tokens) {
    const int32_t rc = check_shape(s);
    if (rc != GDN_OK) return rc;
    if (n_req < 0 || total_tokens < 0) return GDN_ERR_COUNT;
    return plan_bytes(n_req, total_tokens, s->H_q / s->H_kv) + part_ml_bytes() + part_o_bytes(s->d);
}

// shared by attn_kv_restore and attn_kv_spill: rows [0, n_rows[r]) of one pool's slot to the other's
static int32_t kv_tier_copy(const attn_shape* s, int32_t n_req, const int32_t* n_rows, void* host_k, void* host_v,
                            int64_t host_slot_stride, int32_t n_host_slots, const int32_t* host_slot, void* k_cache, void* v_cache,
                            int64_t slot_stride, int32_t n_slots, int32_t cap, const int32_t* seq_slot, bool to_device,
                            hipStream_t stream) {
    int32_t rc = check_shape(s);
    if (rc != GDN_OK) return rc;
    if (n_req < 0 || n_host_slots < 0) return GDN_ERR_COUNT;
    rc = check_pool(s, slot_stride, n_slots, cap);
    if (rc != GDN_OK) return rc;
    rc = check_pool(s, host_slot_stride, n_host_slots, cap);
    if (rc != GDN_OK) return rc;
    if (n_req == 0) return GDN_OK;
    if (!n_rows || !host_slot || !seq_slot) return GDN_ERR_NULL;
    int64_t total = 0;
    for (int32_t r = 0; r < n_req; ++r) {
        if (n_rows[r] < 0 || n_rows[r] > cap) return GDN_ERR_START;
        total += n_rows[r];
    }
    // the source slots only have to exist; the destination slots must also differ
    for (int32_t r = 0; r < n_req; ++r) {
        if (host_slot[r] < 0 || host_slot[r] >= n_host_slots) return GDN_ERR_SLOT_RANGE;
        if (seq_slot[r] < 0 || seq_slot[r] >= n_slots) return GDN_ERR_SLOT_RANGE;
    }
    rc = to_device ? check_slots(seq_slot, n_req, n_slots, false, nullptr) : check_slots(host_slot, n_req, n_host_slots, false, nullptr);
    if (rc != GDN_OK) return rc;
    if (total == 0) return GDN_OK;
    if (!host_k || !host_v || !k_cache || !v_cache) return GDN_ERR_NULL;
    if (!aligned16(k_cache) || !aligned16(v_cache)) return GDN_ERR_ALIGN;
    const int64_t row = (int64_t)s->H_kv * s->d;
    for (int32_t r = 0; r < n_req; ++r) {
        if (n_rows[r] == 0) continue;
        const size_t bytes = (size_t)n_rows[r] * row * sizeof(uint16_t);
        const int64_t ho = (int64_t)host_slot[r] * host_slot_stride, dv = (int64_t)seq_slot[r] * slot_stride;
        uint16_t* const hk = static_cast<uint16_t*>(host_k) + ho;
        uint16_t* const hv = static_cast<uint16_t*>(host_v) + ho;
        uint16_t* const dk = static_cast<uint16_t*>(k_cache) + dv;
        uint16_t* const dvp = static_cast<uint16_t*>(v_cache) + dv;
        hipError_t e = to_device ? hipMemcpyAsync(dk, hk, bytes, hipMemcpyHostToDevice, stream)
                                 : hipMemcpyAsync(hk, dk, bytes, hipMemcpyDeviceToHost, stream);
        if (e != hipSuccess) return hip_err(e);
        e = to_device ? hipMemcpyAsync(dvp, hv, bytes, hipMemcpyHostToDevice, stream)
                      : hipMemcpyAsync(hv, dvp, bytes, hipMemcpyDeviceToHost, stream);
        if (e != hipSuccess) return hip_err(e);
    }
    return GDN_OK;
}

int32_t attn_kv_restore(const attn_shape* s, int32_t n_req, const int32_t* prefix_len, const void* host_k, const void* host_v,
                        int64_t host_slot_stride, int32_t n_host_slots, const int32_t* host_slot, void* k_cache, void* v_cache,
                        int64_t slot_stride, int32_t n_slots, int32_t cap, const int32_t* seq_slot, void* stream) {
    return kv_tier_copy(s, n_req, prefix_len, const_cast<void*>(host_k), const_cast<void*>(host_v), host_slot_stride, n_host_slots,
                        host_slot, k_cache, v_cache, slot_stride, n_slots, cap, seq_slot, true, static_cast<hipStream_t>(stream));
}

int32_t attn_kv_spill(const attn_shape* s, int32_t n_req, const int32_t* n_rows, void* host_k, void* host_v,
                      int64_t host_slot_stride, int32_t n_host_slots, const int32_t* host_slot, const void* k_cache,
                      const void* v_cache, int64_t slot_stride, int32_t n_slots, int32_t cap, const int32_t* seq_slot, void* stream) {
    return kv_tier_copy(s, n_req, n_rows, host_k, host_v, host_slot_stride, n_host_slots, host_slot, const_cast<void*>(k_cache),
                        const_cast<void*>(v_cache), slot_stride, n_slots, cap, seq_slot, false, static_cast<hipStream_t>(stream));
}

int32_t attn_plan(const attn_shape* s, int32_t n_req, const int32_t* cu_seqlens, const int32_t* start_pos, int32_t capacity,
                  int32_t* unit_req, int32_t* unit_tile, int32_t* unit_t0, int32_t* unit_t1, int32_t* unit_part,
                  int32_t* n_units, int32_t* heads_per_row_group, int32_t* key_tile_rows) {
    const int32_t rc = check_shape(s);
    if (rc != GDN_OK) return rc;
    if (n_req < 0 || capacity < 0) return GDN_ERR_COUNT;
    if (!n_units || !heads_per_row_group || !key_tile_rows) return GDN_ERR_NULL;
    *n_units = 0;
    *heads_per_row_group = 1;
    *key_tile_rows = att_kt(s->d);
    if (n_req == 0) return GDN_OK;
    if (!cu_seqlens || !start_pos) return GDN_ERR_NULL;
    if (cu_seqlens[0] != 0) return GDN_ERR_SEQLENS;
    std::vector<int32_t> len(n_req);
    for (int32_t r = 0; r < n_req; ++r) {
        if (cu_seqlens[r + 1] < cu_seqlens[r]) return GDN_ERR_SEQLENS;
        len[r] = cu_seqlens[r + 1] - cu_seqlens[r];
        if (start_pos[r] < 0 || (int64_t)start_pos[r] + len[r] > INT32_MAX - 256) return GDN_ERR_START;
    }
    UnitPlan plan;
    build_units(*s, n_req, len.data(), start_pos, plan);
    *n_units = (int32_t)plan.units.size();
    *heads_per_row_group = plan.pack;
    if ((int64_t)plan.units.size() > capacity) return GDN_ERR_COUNT;
    if (!plan.units.empty() && (!unit_req || !unit_tile || !unit_t0 || !unit_t1 || !unit_part)) return GDN_ERR_NULL;
    for (size_t i = 0; i < plan.units.size(); ++i) {
        unit_req[i] = plan.units[i].req;
        unit_tile[i] = plan.units[i].tile;
        unit_t0[i] = plan.units[i].t0;
        unit_t1[i] = plan.units[i].t1;
        unit_part[i] = plan.units[i].part;
    }
    return GDN_OK;
}

int32_t attn_suffix_prefill(const attn_shape* s, const void* q, const void* k_new, const void* v_new, const void* out_gate,
                            int32_t n_req, const int32_t* cu_seqlens, const int32_t* start_pos, void* k_cache, void* v_cache,
                            int64_t slot_stride, int32_t n_slots, int32_t cap, const int32_t* seq_slot, void* o, void* workspace,
                            int64_t workspace_bytes, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    int32_t rc = check_shape(s);
    if (rc != GDN_OK) return rc;
    if (n_req < 0) return GDN_ERR_COUNT;
    rc = check_pool(s, slot_stride, n_slots, cap);
    if (rc != GDN_OK) return rc;
    if (n_req == 0) return GDN_OK;
    if (!cu_seqlens || !start_pos || !seq_slot) return GDN_ERR_NULL;
    if (cu_seqlens[0] != 0) return GDN_ERR_SEQLENS;
    std::vector<int32_t> len(n_req);
    for (int32_t r = 0; r < n_req; ++r) {
        if (cu_seqlens[r + 1] < cu_seqlens[r]) return GDN_ERR_SEQLENS;
        len[r] = cu_seqlens[r + 1] - cu_seqlens[r];
        if (start_pos[r] < 0 || (int64_t)start_pos[r] + len[r] > cap) return GDN_ERR_START;
    }
    rc = check_slots(seq_slot, n_req, n_slots, true, len.data());
    if (rc != GDN_OK) return rc;
    const int64_t T = cu_seqlens[n_req];
    if (T == 0) return GDN_OK;
    if (!q || !k_new || !v_new || !k_cache || !v_cache || !o) return GDN_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(o) ||
        !aligned16(out_gate))
        return GDN_ERR_ALIGN;
    if (!workspace || !aligned16(workspace) || workspace_bytes < attn_workspace_bytes(s, n_req, T)) return GDN_ERR_WORKSPACE;

    UnitPlan plan;
    build_units(*s, n_req, len.data(), start_pos, plan);
    const int G = s->H_q / s->H_kv;
    const int pack = plan.pack, HB = s->H_q / pack;
    const std::vector<Unit>& units = plan.units;
    const std::vector<int32_t>&piece_req = plan.piece_req, &piece_tile = plan.piece_tile, &piece_base = plan.piece_base,
                              &piece_parts = plan.piece_parts;
    const int64_t n_units = (int64_t)units.size();
    const int64_t n_pieces = (int64_t)piece_req.size();
    const bool xcd_split = 8 % s->H_kv == 0;
    int64_t blocks;
    if (xcd_split) {
        const int X = 8 / s->H_kv;
        blocks = 8 * ((n_units * (G / pack) + X - 1) / X);
    } else {
        blocks = n_units * HB;
    }
    if (blocks > INT32_MAX) return GDN_ERR_COUNT;

    // the uploaded image is packed to what this call uses (the workspace is sized for the most a call can need):
    // a copy of a few hundred bytes takes the runtime's short path, one of 16 KiB and more does not
    const int64_t MU = n_units, MI = n_pieces;
    std::vector<int32_t> img((size_t)(3 * (int64_t)n_req + 1 + 5 * MU + 4 * MI), 0);
    int32_t* p_cu = img.data();
    int32_t* p_start = p_cu + n_req + 1;
    int32_t* p_slot = p_start + n_req;
    int32_t* p_unit = p_slot + n_req;          // five arrays of n_units
    int32_t* p_piece = p_unit + 5 * MU;        // four arrays of n_pieces
    std::memcpy(p_cu, cu_seqlens, sizeof(int32_t) * (n_req + 1));
    std::memcpy(p_start, start_pos, sizeof(int32_t) * n_req);
    std::memcpy(p_slot, seq_slot, sizeof(int32_t) * n_req);
    for (int64_t i = 0; i < n_units; ++i) {
        p_unit[i] = units[i].req;
        p_unit[MU + i] = units[i].tile;
        p_unit[2 * MU + i] = units[i].t0;
        p_unit[3 * MU + i] = units[i].t1;
        p_unit[4 * MU + i] = units[i].part;
    }
    for (int64_t i = 0; i < n_pieces; ++i) {
        p_piece[i] = piece_req[i];
        p_piece[MI + i] = piece_tile[i];
        p_piece[2 * MI + i] = piece_base[i];
        p_piece[3 * MI + i] = piece_parts[i];
    }
    rc = gdn::upload_plan(img.data(), img.size() * sizeof(int32_t), workspace, stream);
    if (rc != GDN_OK) return rc;
    const int32_t* d = static_cast<const int32_t*>(workspace);

    AppendArgs ap;
    ap.k_new = static_cast<const uint16_t*>(k_new);
    ap.v_new = static_cast<const uint16_t*>(v_new);
    ap.k_cache = static_cast<uint16_t*>(k_cache);
    ap.v_cache = static_cast<uint16_t*>(v_cache);
    ap.cu = d;
    ap.start = d + n_req + 1;
    ap.slot = d + 2 * (int64_t)n_req + 1;
    ap.slot_stride = slot_stride;
    ap.row_chunks = s->H_kv * s->d / 8;
    ap.n_chunks = T * ap.row_chunks;
    ap.n_req = n_req;
    const int64_t ablocks = (ap.n_chunks + APPEND_THREADS - 1) / APPEND_THREADS;
    if (ablocks > INT32_MAX) return GDN_ERR_COUNT;
    hipLaunchKernelGGL(attn_append_kernel, dim3((unsigned)ablocks), dim3(APPEND_THREADS), 0, stream, ap);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_err(e);

    AttnArgs a;
    a.q = static_cast<const uint16_t*>(q);
    a.gate = static_cast<const uint16_t*>(out_gate);
    a.k_cache = ap.k_cache;
    a.v_cache = ap.v_cache;
    a.o = o;
    a.cu = ap.cu;
    a.start = ap.start;
    a.slot = ap.slot;
    a.unit_req = d + 3 * (int64_t)n_req + 1;
    a.unit_tile = a.unit_req + MU;
    a.unit_t0 = a.unit_req + 2 * MU;
    a.unit_t1 = a.unit_req + 3 * MU;
    a.unit_part = a.unit_req + 4 * MU;
    a.part_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + plan_bytes(n_req, T, G));
    a.part_o = reinterpret_cast<float*>(static_cast<char*>(workspace) + plan_bytes(n_req, T, G) + part_ml_bytes());
    a.slot_stride = slot_stride;
    a.n_units = (int32_t)n_units;
    a.H_q = s->H_q;
    a.H_kv = s->H_kv;
    a.xcd_split = xcd_split ? 1 : 0;
    a.pack = pack;
    a.scale_log2e = s->scale * 1.4426950408889634f;
    e = s->o_dtype == GDN_F32 ? launch_attn_d<float>(s->d, a, (unsigned)blocks, stream)
                              : launch_attn_d<uint16_t>(s->d, a, (unsigned)blocks, stream);
    if (e != hipSuccess || n_pieces == 0) return hip_err(e);

    CombineArgs ca;
    ca.part_o = a.part_o;
    ca.part_ml = a.part_ml;
    ca.gate = a.gate;
    ca.o = o;
    ca.cu = a.cu;
    ca.piece_req = a.unit_req + 5 * MU;
    ca.piece_tile = ca.piece_req + MI;
    ca.piece_base = ca.piece_req + 2 * MI;
    ca.piece_parts = ca.piece_req + 3 * MI;
    ca.H_q = s->H_q;
    ca.pack = pack;
    ca.scale_log2e = a.scale_log2e;
    e = s->o_dtype == GDN_F32 ? launch_combine_d<float>(s->d, ca, (unsigned)(n_pieces * HB), stream)
                              : launch_combine_d<uint16_t>(s->d, ca, (unsigned)(n_pieces * HB), stream);
    return hip_err(e);
}

int32_t attn_tune_split(int32_t allow) { return g_allow_split.exchange(allow != 0); }

int32_t attn_tune_pack(int32_t allow) { return g_allow_pack.exchange(allow != 0); }

}  // extern "C"
