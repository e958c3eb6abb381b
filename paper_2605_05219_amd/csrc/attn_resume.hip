// attn_resume: host side of the attention layers' part of a cache hit (see include/attn_resume.h).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
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

// ints of the uploaded index arrays: cu (n_req+1), start, slot (n_req each), item_req, item_tile
inline int64_t max_items(int32_t n_req, int64_t T) { return T / ATT_BQ + n_req; }
inline int64_t plan_ints(int32_t n_req, int64_t T) { return 3 * (int64_t)n_req + 1 + 2 * max_items(n_req, T); }

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

}  // namespace
}  // namespace attn

using namespace attn;

extern "C" {

int64_t attn_workspace_bytes(int32_t n_req, int64_t total_tokens) {
    if (n_req < 0 || total_tokens < 0) return GDN_ERR_COUNT;
    return (plan_ints(n_req, total_tokens) * (int64_t)sizeof(int32_t) + 255) / 256 * 256;
}

int32_t attn_kv_restore(const attn_shape* s, int32_t n_req, const int32_t* prefix_len, const void* host_k, const void* host_v,
                        int64_t host_slot_stride, int32_t n_host_slots, const int32_t* host_slot, void* k_cache, void* v_cache,
                        int64_t slot_stride, int32_t n_slots, int32_t cap, const int32_t* seq_slot, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    int32_t rc = check_shape(s);
    if (rc != GDN_OK) return rc;
    if (n_req < 0 || n_host_slots < 0) return GDN_ERR_COUNT;
    rc = check_pool(s, slot_stride, n_slots, cap);
    if (rc != GDN_OK) return rc;
    rc = check_pool(s, host_slot_stride, n_host_slots, cap);
    if (rc != GDN_OK) return rc;
    if (n_req == 0) return GDN_OK;
    if (!prefix_len || !host_slot || !seq_slot) return GDN_ERR_NULL;
    int64_t total = 0;
    for (int32_t r = 0; r < n_req; ++r) {
        if (prefix_len[r] < 0 || prefix_len[r] > cap) return GDN_ERR_START;
        if (host_slot[r] < 0 || host_slot[r] >= n_host_slots) return GDN_ERR_SLOT_RANGE;
        total += prefix_len[r];
    }
    rc = check_slots(seq_slot, n_req, n_slots, false, nullptr);
    if (rc != GDN_OK) return rc;
    if (total == 0) return GDN_OK;
    if (!host_k || !host_v || !k_cache || !v_cache) return GDN_ERR_NULL;
    if (!aligned16(k_cache) || !aligned16(v_cache)) return GDN_ERR_ALIGN;
    const int64_t row = (int64_t)s->H_kv * s->d;
    for (int32_t r = 0; r < n_req; ++r) {
        if (prefix_len[r] == 0) continue;
        const size_t bytes = (size_t)prefix_len[r] * row * sizeof(uint16_t);
        const int64_t src = (int64_t)host_slot[r] * host_slot_stride, dst = (int64_t)seq_slot[r] * slot_stride;
        hipError_t e = hipMemcpyAsync(static_cast<uint16_t*>(k_cache) + dst, static_cast<const uint16_t*>(host_k) + src, bytes,
                                      hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) return hip_err(e);
        e = hipMemcpyAsync(static_cast<uint16_t*>(v_cache) + dst, static_cast<const uint16_t*>(host_v) + src, bytes,
                           hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) return hip_err(e);
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
    if (!workspace || !aligned16(workspace) || workspace_bytes < attn_workspace_bytes(n_req, T)) return GDN_ERR_WORKSPACE;

    // ---- work items: one per 128 suffix tokens of a request, those that see the most keys first
    struct Item { int32_t req, tile, kv; };
    std::vector<Item> items;
    for (int32_t r = 0; r < n_req; ++r)
        for (int32_t t = 0; t * ATT_BQ < len[r]; ++t)
            items.push_back({r, t, start_pos[r] + std::min((t + 1) * ATT_BQ, len[r])});
    std::stable_sort(items.begin(), items.end(), [](const Item& x, const Item& y) { return x.kv > y.kv; });
    const int64_t n_items = (int64_t)items.size();
    const int G = s->H_q / s->H_kv;
    const bool xcd_split = 8 % s->H_kv == 0;
    int64_t blocks;
    if (xcd_split) {
        const int X = 8 / s->H_kv;
        blocks = 8 * ((n_items * G + X - 1) / X);
    } else {
        blocks = n_items * s->H_q;
    }
    if (blocks > INT32_MAX) return GDN_ERR_COUNT;

    std::vector<int32_t> img((size_t)plan_ints(n_req, T), 0);
    int32_t* p_cu = img.data();
    int32_t* p_start = p_cu + n_req + 1;
    int32_t* p_slot = p_start + n_req;
    int32_t* p_ireq = p_slot + n_req;
    int32_t* p_itile = p_ireq + max_items(n_req, T);
    std::memcpy(p_cu, cu_seqlens, sizeof(int32_t) * (n_req + 1));
    std::memcpy(p_start, start_pos, sizeof(int32_t) * n_req);
    std::memcpy(p_slot, seq_slot, sizeof(int32_t) * n_req);
    for (int64_t i = 0; i < n_items; ++i) {
        p_ireq[i] = items[i].req;
        p_itile[i] = items[i].tile;
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
    a.item_req = d + 3 * (int64_t)n_req + 1;
    a.item_tile = a.item_req + max_items(n_req, T);
    a.slot_stride = slot_stride;
    a.n_items = (int32_t)n_items;
    a.H_q = s->H_q;
    a.H_kv = s->H_kv;
    a.xcd_split = xcd_split ? 1 : 0;
    a.scale_log2e = s->scale * 1.4426950408889634f;
    e = s->o_dtype == GDN_F32 ? launch_attn_d<float>(s->d, a, (unsigned)blocks, stream)
                              : launch_attn_d<uint16_t>(s->d, a, (unsigned)blocks, stream);
    return hip_err(e);
}

}  // extern "C"
