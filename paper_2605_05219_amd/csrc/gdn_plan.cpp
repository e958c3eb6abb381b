// Host-side planning and validation for the resume prefill (integer work only).
#include "gdn_plan.h"

#include <algorithm>
#include <numeric>

namespace gdn {

int32_t check_shape(const gdn_shape* s) {
    if (!s) return GDN_ERR_NULL;
    if (s->L <= 0 || s->H_qk <= 0 || s->H_v <= 0) return GDN_ERR_SHAPE;
    if (s->H_v % s->H_qk != 0) return GDN_ERR_SHAPE;
    if (!((s->d_k == 64 && s->d_v == 64) || (s->d_k == 128 && s->d_v == 128))) return GDN_ERR_SHAPE;
    if (s->in_dtype != GDN_F32 && s->in_dtype != GDN_BF16) return GDN_ERR_SHAPE;
    if (s->o_dtype != GDN_F32 && s->o_dtype != GDN_BF16) return GDN_ERR_SHAPE;
    if (s->in_dtype == GDN_F32 && s->d_k != 64) return GDN_ERR_SHAPE;  // fp32 inputs: d = 64 only
    if (s->T_alloc < 0) return GDN_ERR_SHAPE;
    if (!(s->scale == s->scale)) return GDN_ERR_SHAPE;
    return GDN_OK;
}

int32_t plan_chunks(int32_t n_req, const int32_t* cu, const int32_t* start_pos,
                    const int32_t* emit_cu, const int32_t* emit_pos, ChunkPlan* out) {
    if (n_req < 0) return GDN_ERR_COUNT;
    if (!cu || !emit_cu || !out) return GDN_ERR_NULL;
    if (n_req > 0 && !start_pos) return GDN_ERR_NULL;
    if (cu[0] != 0) return GDN_ERR_SEQLENS;
    if (emit_cu[0] != 0) return GDN_ERR_EMIT;
    for (int32_t r = 0; r < n_req; ++r) {
        if (cu[r + 1] < cu[r]) return GDN_ERR_SEQLENS;
        if (emit_cu[r + 1] < emit_cu[r]) return GDN_ERR_EMIT;
    }
    if (emit_cu[n_req] > 0 && !emit_pos) return GDN_ERR_NULL;

    out->chunk_tok0.clear();
    out->chunk_len.clear();
    out->chunk_emit.clear();
    out->req_chunk_cu.assign(1, 0);
    out->max_chunks_per_req = 0;

    for (int32_t r = 0; r < n_req; ++r) {
        const int64_t len = (int64_t)cu[r + 1] - cu[r];
        const int64_t l = start_pos[r];
        if (l < 0) return GDN_ERR_START;
        if (l + len > INT32_MAX) return GDN_ERR_START;
        int64_t prev = l;  // absolute position reached so far
        int32_t tok = cu[r];
        auto cut = [&](int64_t upto, int32_t emit_idx) {
            // chunks covering absolute positions (prev, upto]; the last one carries the emission
            while (prev < upto) {
                const int32_t n = (int32_t)std::min<int64_t>(GDN_CHUNK, upto - prev);
                prev += n;
                out->chunk_tok0.push_back(tok);
                out->chunk_len.push_back(n);
                out->chunk_emit.push_back(prev == upto ? emit_idx : -1);
                tok += n;
            }
        };
        for (int32_t e = emit_cu[r]; e < emit_cu[r + 1]; ++e) {
            const int64_t p = emit_pos[e];
            if (p <= prev || p > l + len) return GDN_ERR_EMIT;  // strictly increasing, in (l, end]
            cut(p, e);
        }
        cut(l + len, -1);
        const int32_t first = out->req_chunk_cu.back();
        const int32_t last = (int32_t)out->chunk_tok0.size();
        out->req_chunk_cu.push_back(last);
        out->max_chunks_per_req = std::max(out->max_chunks_per_req, last - first);
    }
    return GDN_OK;
}

int32_t check_slots(int32_t n_req, const int32_t* src_slot, int32_t src_n_slots,
                    const int32_t* emit_cu, const int32_t* emit_slot, int32_t dst_n_slots) {
    if (n_req > 0 && !src_slot) return GDN_ERR_NULL;
    if (src_n_slots < 0 || dst_n_slots < 0) return GDN_ERR_COUNT;
    for (int32_t r = 0; r < n_req; ++r)
        if (src_slot[r] < -1 || src_slot[r] >= src_n_slots) return GDN_ERR_SLOT_RANGE;
    const int32_t n_emit = emit_cu[n_req];
    if (n_emit > 0 && !emit_slot) return GDN_ERR_NULL;
    std::vector<int32_t> dst(emit_slot, emit_slot + n_emit);
    for (int32_t id : dst)
        if (id < 0 || id >= dst_n_slots) return GDN_ERR_SLOT_RANGE;
    std::sort(dst.begin(), dst.end());
    if (std::adjacent_find(dst.begin(), dst.end()) != dst.end()) return GDN_ERR_SLOT_DUP;
    return GDN_OK;
}

std::vector<int32_t> longest_first(const ChunkPlan& plan, int32_t n_req) {
    std::vector<int32_t> order(n_req);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return plan.req_chunk_cu[a + 1] - plan.req_chunk_cu[a] > plan.req_chunk_cu[b + 1] - plan.req_chunk_cu[b];
    });
    return order;
}

}  // namespace gdn
