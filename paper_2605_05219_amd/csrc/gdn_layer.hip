// gdn_layer: host side of the layer's elementwise front and back ends (see include/gdn_layer.h).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <vector>

#include "gdn_host.h"
#include "gdn_layer.h"
#include "gdn_layer_kernel.h"

namespace gdn {
namespace {

inline int32_t hip_err(hipError_t e) { return e == hipSuccess ? GDN_OK : GDN_ERR_HIP - (int32_t)e; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool dtype_ok(int32_t t) { return t == GDN_F32 || t == GDN_BF16; }
inline int elem_bytes(int32_t t) { return t == GDN_F32 ? 4 : 2; }

int32_t check_shape(const gdn_layer_shape* s) {
    if (!s) return GDN_ERR_NULL;
    if (s->H_qk <= 0 || s->H_v <= 0 || s->L <= 0 || s->T_alloc < 0) return GDN_ERR_SHAPE;
    if ((s->d_k != 64 && s->d_k != 128) || (s->d_v != 64 && s->d_v != 128)) return GDN_ERR_SHAPE;
    if (s->conv_k < 2 || s->conv_k > 4) return GDN_ERR_SHAPE;
    if (!dtype_ok(s->in_dtype) || !dtype_ok(s->out_dtype) || !dtype_ok(s->o_dtype)) return GDN_ERR_SHAPE;
    if (!(s->qk_eps >= 0.f) || !(s->norm_eps >= 0.f)) return GDN_ERR_SHAPE;
    // the lanes of a q/k head must not straddle a row of channel groups
    if (((int64_t)s->H_v * s->d_v) % s->d_k != 0) return GDN_ERR_SHAPE;
    return GDN_OK;
}

// ints of the uploaded index arrays: cu (n_req+1), start, src_slot (n_req each), run_cu (n_req+1),
// emit_req, emit_pos, emit_slot (n_emit each)
inline int64_t plan_ints(int32_t n_req, int32_t n_emit) { return 4 * (int64_t)n_req + 2 + 3 * (int64_t)n_emit; }

template <typename In, typename Out>
hipError_t launch_inputs(const LayerArgs& a, int64_t blocks, int layers, hipStream_t stream) {
    hipLaunchKernelGGL((gdn_layer_inputs_kernel<In, Out>), dim3((unsigned)blocks, (unsigned)layers), dim3(LAYER_THREADS), 0, stream, a);
    return hipGetLastError();
}

template <typename O, typename In, typename Out>
hipError_t launch_output(const LayerOutArgs& a, int64_t blocks, int layers, hipStream_t stream) {
    hipLaunchKernelGGL((gdn_layer_output_kernel<O, In, Out>), dim3((unsigned)blocks, (unsigned)layers), dim3(LAYER_THREADS), 0, stream, a);
    return hipGetLastError();
}

}  // namespace
}  // namespace gdn

using namespace gdn;

extern "C" {

int64_t gdn_layer_workspace_bytes(int32_t n_req, int32_t n_emit) {
    if (n_req < 0 || n_emit < 0) return GDN_ERR_COUNT;
    return (plan_ints(n_req, n_emit) * (int64_t)sizeof(int32_t) + 255) / 256 * 256;
}

int32_t gdn_layer_inputs(const gdn_layer_shape* s, const void* x_qkv, const float* conv_w, const float* conv_b,
                         const void* a_pre, const void* b_pre, const float* A_log, const float* dt_bias, int32_t n_req,
                         const int32_t* cu_seqlens, const int32_t* start_pos, const void* conv_src,
                         int64_t src_slot_stride, int32_t n_src_slots, const int32_t* src_slot, const int32_t* emit_cu,
                         const int32_t* emit_pos, void* conv_dst, int64_t dst_slot_stride, int32_t n_dst_slots,
                         const int32_t* emit_slot, void* q, void* k, void* v, void* beta, void* gate, void* workspace,
                         int64_t workspace_bytes, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    int32_t rc = check_shape(s);
    if (rc != GDN_OK) return rc;
    if (n_req < 0 || n_src_slots < 0 || n_dst_slots < 0) return GDN_ERR_COUNT;
    if (n_req == 0) return GDN_OK;
    if (!cu_seqlens || !start_pos || !src_slot || !emit_cu) return GDN_ERR_NULL;
    // ---- index arrays
    if (cu_seqlens[0] != 0 || emit_cu[0] != 0) return GDN_ERR_SEQLENS;
    for (int32_t r = 0; r < n_req; ++r) {
        if (cu_seqlens[r + 1] < cu_seqlens[r] || emit_cu[r + 1] < emit_cu[r]) return GDN_ERR_SEQLENS;
        if (start_pos[r] < 0 || (int64_t)start_pos[r] + (cu_seqlens[r + 1] - cu_seqlens[r]) > INT32_MAX) return GDN_ERR_START;
    }
    const int64_t T = cu_seqlens[n_req];
    if (s->T_alloc && T > s->T_alloc) return GDN_ERR_SEQLENS;
    const int32_t n_emit = emit_cu[n_req];
    if (n_emit > 0 && (!emit_pos || !emit_slot)) return GDN_ERR_NULL;
    const int32_t K1 = s->conv_k - 1;
    const int64_t C = 2 * (int64_t)s->H_qk * s->d_k + (int64_t)s->H_v * s->d_v;
    if (C > (1 << 24)) return GDN_ERR_SHAPE;
    std::vector<int32_t> emit_req((size_t)n_emit);
    for (int32_t r = 0; r < n_req; ++r) {
        const int32_t end = start_pos[r] + (cu_seqlens[r + 1] - cu_seqlens[r]);
        int32_t prev = start_pos[r];
        for (int32_t e = emit_cu[r]; e < emit_cu[r + 1]; ++e) {
            if (emit_pos[e] <= prev || emit_pos[e] > end) return GDN_ERR_EMIT;
            prev = emit_pos[e];
            emit_req[(size_t)e] = r;
        }
    }
    bool any_src = false;
    for (int32_t r = 0; r < n_req; ++r) {
        if (src_slot[r] < -1 || src_slot[r] >= n_src_slots) return GDN_ERR_SLOT_RANGE;
        any_src = any_src || src_slot[r] >= 0;
    }
    {
        std::vector<int32_t> sorted(emit_slot, emit_slot + n_emit);
        for (int32_t id : sorted)
            if (id < 0 || id >= n_dst_slots) return GDN_ERR_SLOT_RANGE;
        std::sort(sorted.begin(), sorted.end());
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return GDN_ERR_SLOT_DUP;
    }
    if (n_emit > 0 && any_src && conv_src && conv_dst) {
        // by address (the pools may be the same memory under different base pointers): no destination slot may
        // overlap a source slot that this launch reads
        const uintptr_t eb = (uintptr_t)elem_bytes(s->in_dtype), bytes = (uintptr_t)s->L * K1 * C * eb;
        std::vector<uintptr_t> dlo((size_t)n_emit);
        for (int32_t e = 0; e < n_emit; ++e)
            dlo[(size_t)e] = reinterpret_cast<uintptr_t>(conv_dst) + (uintptr_t)emit_slot[e] * (uintptr_t)dst_slot_stride * eb;
        std::sort(dlo.begin(), dlo.end());
        for (int32_t r = 0; r < n_req; ++r) {
            if (src_slot[r] < 0) continue;
            const uintptr_t lo = reinterpret_cast<uintptr_t>(conv_src) + (uintptr_t)src_slot[r] * (uintptr_t)src_slot_stride * eb;
            auto it = std::upper_bound(dlo.begin(), dlo.end(), lo);
            if (it != dlo.begin() && *(it - 1) + bytes > lo) return GDN_ERR_SLOT_HAZARD;
            if (it != dlo.end() && *it < lo + bytes) return GDN_ERR_SLOT_HAZARD;
        }
    }
    // ---- pointers
    if (T > 0 && (!x_qkv || !conv_w || !a_pre || !b_pre || !A_log || !dt_bias || !q || !k || !v || !beta || !gate))
        return GDN_ERR_NULL;
    if ((any_src && !conv_src) || (n_emit > 0 && !conv_dst)) return GDN_ERR_NULL;
    const void* ptrs[] = {x_qkv, conv_w, conv_b, a_pre, b_pre, conv_src, conv_dst, q, k, v, beta, gate};
    for (const void* p : ptrs)
        if (!aligned16(p)) return GDN_ERR_ALIGN;
    const int64_t per16 = 16 / elem_bytes(s->in_dtype);
    if (any_src) {
        if (src_slot_stride % per16) return GDN_ERR_ALIGN;
        if (src_slot_stride < (int64_t)s->L * K1 * C) return GDN_ERR_SHAPE;
    }
    if (n_emit > 0) {
        if (dst_slot_stride % per16) return GDN_ERR_ALIGN;
        if (dst_slot_stride < (int64_t)s->L * K1 * C) return GDN_ERR_SHAPE;
    }
    const int64_t need = gdn_layer_workspace_bytes(n_req, n_emit);
    if (!workspace || !aligned16(workspace) || workspace_bytes < need) return GDN_ERR_WORKSPACE;

    // ---- plan: [cu | start | src_slot | run_cu | emit_req | emit_pos | emit_slot]
    std::vector<int32_t> plan((size_t)plan_ints(n_req, n_emit));
    int32_t* p_cu = plan.data();
    int32_t* p_start = p_cu + n_req + 1;
    int32_t* p_src = p_start + n_req;
    int32_t* p_run = p_src + n_req;
    int32_t* p_ereq = p_run + n_req + 1;
    int32_t* p_epos = p_ereq + n_emit;
    int32_t* p_eslot = p_epos + n_emit;
    std::memcpy(p_cu, cu_seqlens, sizeof(int32_t) * (n_req + 1));
    std::memcpy(p_start, start_pos, sizeof(int32_t) * n_req);
    std::memcpy(p_src, src_slot, sizeof(int32_t) * n_req);
    int64_t runs = 0;
    for (int32_t r = 0; r < n_req; ++r) {
        p_run[r] = (int32_t)runs;
        runs += (cu_seqlens[r + 1] - cu_seqlens[r] + LAYER_RUN - 1) / LAYER_RUN;
    }
    p_run[n_req] = (int32_t)runs;
    if (n_emit > 0) {
        std::memcpy(p_ereq, emit_req.data(), sizeof(int32_t) * n_emit);
        std::memcpy(p_epos, emit_pos, sizeof(int32_t) * n_emit);
        std::memcpy(p_eslot, emit_slot, sizeof(int32_t) * n_emit);
    }
    const int64_t CG = C / 8;
    const int64_t conv_blocks = (runs * CG + LAYER_THREADS - 1) / LAYER_THREADS;
    const int64_t gate_blocks = (T * s->H_v + LAYER_THREADS - 1) / LAYER_THREADS;
    const int64_t emit_blocks = ((int64_t)n_emit * K1 * CG + LAYER_THREADS - 1) / LAYER_THREADS;
    const int64_t blocks = conv_blocks + gate_blocks + emit_blocks;
    if (blocks > INT32_MAX) return GDN_ERR_COUNT;
    if (blocks == 0) return GDN_OK;
    rc = upload_plan(plan.data(), plan.size() * sizeof(int32_t), workspace, stream);
    if (rc != GDN_OK) return rc;

    LayerArgs a;
    a.x = x_qkv; a.w = conv_w; a.bias = conv_b; a.a_pre = a_pre; a.b_pre = b_pre; a.A_log = A_log; a.dt_bias = dt_bias;
    a.conv_src = conv_src; a.conv_dst = conv_dst; a.src_stride = src_slot_stride; a.dst_stride = dst_slot_stride;
    a.q = q; a.k = k; a.v = v; a.beta = beta; a.gate = gate;
    const int32_t* d = reinterpret_cast<const int32_t*>(workspace);
    a.cu = d; a.start = d + (p_start - p_cu); a.src_slot = d + (p_src - p_cu); a.run_cu = d + (p_run - p_cu);
    a.emit_req = d + (p_ereq - p_cu); a.emit_pos = d + (p_epos - p_cu); a.emit_slot = d + (p_eslot - p_cu);
    a.n_req = n_req; a.n_emit = n_emit; a.n_runs = (int32_t)runs;
    a.C = (int32_t)C; a.nq = s->H_qk * s->d_k; a.d_k = s->d_k; a.H_v = s->H_v; a.K = s->conv_k;
    a.T = T; a.qk_eps = s->qk_eps;
    a.conv_blocks = (int32_t)conv_blocks; a.gate_blocks = (int32_t)gate_blocks;
    const int64_t Tp = s->T_alloc ? s->T_alloc : T;    // tokens per layer plane
    a.ls_x = Tp * C; a.ls_tok_h = Tp * s->H_v; a.ls_qk = Tp * a.nq; a.ls_v = Tp * (C - 2 * a.nq);
    a.ls_w = C * s->conv_k; a.ls_c = C; a.ls_h = s->H_v; a.ls_conv = (int64_t)K1 * C;
    hipError_t e;
    if (s->in_dtype == GDN_BF16)
        e = s->out_dtype == GDN_BF16 ? launch_inputs<uint16_t, uint16_t>(a, blocks, s->L, stream) : launch_inputs<uint16_t, float>(a, blocks, s->L, stream);
    else
        e = s->out_dtype == GDN_BF16 ? launch_inputs<float, uint16_t>(a, blocks, s->L, stream) : launch_inputs<float, float>(a, blocks, s->L, stream);
    return hip_err(e);
}

int32_t gdn_layer_output(const gdn_layer_shape* s, const void* o, const void* z, const float* weight, void* y, int64_t T,
                         void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const int32_t rc = check_shape(s);
    if (rc != GDN_OK) return rc;
    if (T < 0) return GDN_ERR_COUNT;
    if (s->T_alloc && T > s->T_alloc) return GDN_ERR_SEQLENS;
    if (T == 0) return GDN_OK;
    if (!o || !z || !weight || !y) return GDN_ERR_NULL;
    if (!aligned16(o) || !aligned16(z) || !aligned16(weight) || !aligned16(y)) return GDN_ERR_ALIGN;
    LayerOutArgs a;
    a.o = o; a.z = z; a.weight = weight; a.y = y;
    a.n_groups = T * s->H_v * (s->d_v / 8);
    a.d_v = s->d_v;
    a.eps = s->norm_eps;
    a.ls_tok = (s->T_alloc ? s->T_alloc : T) * s->H_v * s->d_v;
    const int64_t blocks = (a.n_groups + LAYER_THREADS - 1) / LAYER_THREADS;
    if (blocks > INT32_MAX) return GDN_ERR_COUNT;
    const int key = (s->o_dtype == GDN_BF16) * 4 + (s->in_dtype == GDN_BF16) * 2 + (s->out_dtype == GDN_BF16);
    hipError_t e = hipSuccess;
    switch (key) {
        case 0: e = launch_output<float, float, float>(a, blocks, s->L, stream); break;
        case 1: e = launch_output<float, float, uint16_t>(a, blocks, s->L, stream); break;
        case 2: e = launch_output<float, uint16_t, float>(a, blocks, s->L, stream); break;
        case 3: e = launch_output<float, uint16_t, uint16_t>(a, blocks, s->L, stream); break;
        case 4: e = launch_output<uint16_t, float, float>(a, blocks, s->L, stream); break;
        case 5: e = launch_output<uint16_t, float, uint16_t>(a, blocks, s->L, stream); break;
        case 6: e = launch_output<uint16_t, uint16_t, float>(a, blocks, s->L, stream); break;
        default: e = launch_output<uint16_t, uint16_t, uint16_t>(a, blocks, s->L, stream); break;
    }
    return hip_err(e);
}

}  // extern "C"
