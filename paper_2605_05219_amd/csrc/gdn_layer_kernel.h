// Elementwise front and back ends of a GatedDeltaNet layer around the resumed recurrence: the
// short convolution continued from its checkpointed state, q/k normalisation, gates, and the
// gated output normalisation (the published layer; the paper's Sec. 1 asks for every part of
// the layer's hidden state to be restored exactly, and the last K-1 convolution inputs are the
// part that is not the matrix state).  All of it is bound by memory traffic: every thread owns
// 8 adjacent channels (16 bytes of bf16) so that a wave reads and writes whole 1 KiB rows, and
// a token run per thread keeps the convolution window in registers so that each input row is
// read once (plus a 3-row halo per run that the neighbouring run has just pulled through L2).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace gdn {

constexpr int LAYER_THREADS = 256;
constexpr int LAYER_RUN = 32;   // tokens per thread of the convolution role

struct LayerArgs {
    const void* x;          // [T][C]
    const float* w;         // [C][K]
    const float* bias;      // [C] or null
    const void* a_pre;      // [T][H_v]
    const void* b_pre;
    const float* A_log;     // [H_v]
    const float* dt_bias;
    const void* conv_src;   // slots of [K-1][C]
    void* conv_dst;
    int64_t src_stride, dst_stride;   // elements
    void *q, *k, *v, *beta, *gate;
    // index arrays in the workspace
    const int32_t* cu;        // n_req + 1
    const int32_t* start;     // n_req
    const int32_t* src_slot;  // n_req
    const int32_t* run_cu;    // n_req + 1: request r owns runs [run_cu[r], run_cu[r+1])
    const int32_t* emit_req;  // n_emit
    const int32_t* emit_pos;  // n_emit (absolute)
    const int32_t* emit_slot; // n_emit
    int32_t n_req, n_emit, n_runs;
    int32_t C, nq, d_k, H_v, K;       // nq = H_qk d_k; channels [0,nq) q, [nq,2nq) k, rest v
    int64_t T;
    float qk_eps;
    int32_t conv_blocks, gate_blocks;  // blocks [0, conv_blocks) convolve, the next gate_blocks make the gates,
                                       // the rest copy convolution states
    // stacked layers (grid.y): element strides from one layer's plane to the next
    int64_t ls_x, ls_tok_h;            // x_qkv; a_pre, b_pre, beta, gate
    int64_t ls_qk, ls_v;               // q and k; v
    int64_t ls_w, ls_c, ls_h;          // taps; bias; A_log and dt_bias
    int64_t ls_conv;                   // a layer's rows inside a convolution-state slot: (K-1) C
};

// ---- 8 adjacent elements <-> fp32
struct F8 { float f[8]; };

__device__ __forceinline__ F8 load8(const uint16_t* p) {   // bf16 bit patterns
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    const uint32_t u[4] = {r.x, r.y, r.z, r.w};
    F8 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o.f[2 * i] = __uint_as_float(u[i] << 16);
        o.f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
    return o;
}
__device__ __forceinline__ F8 load8(const float* p) {
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    return F8{{a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w}};
}
// The same for data that is read once (non-temporal loads).
typedef uint32_t lu32x4 __attribute__((ext_vector_type(4)));
typedef float lf32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ F8 load8_once(const uint16_t* p) {
    const lu32x4 r = __builtin_nontemporal_load(reinterpret_cast<const lu32x4*>(p));
    F8 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o.f[2 * i] = __uint_as_float(r[i] << 16);
        o.f[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
    }
    return o;
}
__device__ __forceinline__ F8 load8_once(const float* p) {
    const lf32x4 a = __builtin_nontemporal_load(reinterpret_cast<const lf32x4*>(p)), b = __builtin_nontemporal_load(reinterpret_cast<const lf32x4*>(p) + 1);
    return F8{{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]}};
}
// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ void store8(uint16_t* p, const F8& v) {
    *reinterpret_cast<uint4*>(p) = make_uint4(pack_bf16(v.f[0], v.f[1]), pack_bf16(v.f[2], v.f[3]), pack_bf16(v.f[4], v.f[5]),
                                              pack_bf16(v.f[6], v.f[7]));
}
__device__ __forceinline__ void store8(float* p, const F8& v) {
    reinterpret_cast<float4*>(p)[0] = make_float4(v.f[0], v.f[1], v.f[2], v.f[3]);
    reinterpret_cast<float4*>(p)[1] = make_float4(v.f[4], v.f[5], v.f[6], v.f[7]);
}
__device__ __forceinline__ float load1(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ void store1(uint16_t* p, float x) { *p = (uint16_t)(pack_bf16(x, 0.f) & 0xffffu); }
__device__ __forceinline__ void store1(float* p, float x) { *p = x; }

__device__ __forceinline__ float silu_f(float x) { return x * __builtin_amdgcn_rcpf(1.f + __expf(-x)); }

// Raw 16-byte-granular loads of 8 elements, widened to fp32 when they are used.
struct Raw16 { uint4 r; };
struct Raw32 { uint4 r[2]; };
__device__ __forceinline__ Raw16 load_raw8(const uint16_t* p) { return Raw16{*reinterpret_cast<const uint4*>(p)}; }
__device__ __forceinline__ Raw32 load_raw8(const float* p) {
    return Raw32{{reinterpret_cast<const uint4*>(p)[0], reinterpret_cast<const uint4*>(p)[1]}};
}
__device__ __forceinline__ F8 widen8(const Raw16& x) {
    const uint32_t u[4] = {x.r.x, x.r.y, x.r.z, x.r.w};
    F8 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o.f[2 * i] = __uint_as_float(u[i] << 16);
        o.f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
    return o;
}
__device__ __forceinline__ F8 widen8(const Raw32& x) {
    return F8{{__uint_as_float(x.r[0].x), __uint_as_float(x.r[0].y), __uint_as_float(x.r[0].z), __uint_as_float(x.r[0].w),
               __uint_as_float(x.r[1].x), __uint_as_float(x.r[1].y), __uint_as_float(x.r[1].z), __uint_as_float(x.r[1].w)}};
}

// Sum over the d/8 adjacent lanes that hold one head (8 lanes for d = 64, 16 for d = 128), every
// lane receiving the total: four cross-lane adds inside a 16-lane row (lane ^ 1, lane ^ 2, then
// the mirror image inside 8 lanes and inside 16 lanes), no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float s) {
    return s + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float head_sum(float s, int d) {
    s = dpp_add<0xB1>(s);    // quad_perm [1,0,3,2]
    s = dpp_add<0x4E>(s);    // quad_perm [2,3,0,1]
    s = dpp_add<0x141>(s);   // row_half_mirror: lane i <-> 7 - i of each 8
    if (d == 128) s = dpp_add<0x140>(s);   // row_mirror: lane i <-> 15 - i of each 16
    return s;
}

template <typename In, typename Out>
__global__ void __launch_bounds__(LAYER_THREADS) gdn_layer_inputs_kernel(LayerArgs a) {
    {   // this block's layer: every tensor moves to that layer's plane
        const int64_t l = blockIdx.y;
        a.x = reinterpret_cast<const In*>(a.x) + l * a.ls_x;
        a.a_pre = reinterpret_cast<const In*>(a.a_pre) + l * a.ls_tok_h;
        a.b_pre = reinterpret_cast<const In*>(a.b_pre) + l * a.ls_tok_h;
        a.w += l * a.ls_w;
        if (a.bias) a.bias += l * a.ls_c;
        a.A_log += l * a.ls_h;
        a.dt_bias += l * a.ls_h;
        if (a.conv_src) a.conv_src = reinterpret_cast<const In*>(a.conv_src) + l * a.ls_conv;
        if (a.conv_dst) a.conv_dst = reinterpret_cast<In*>(a.conv_dst) + l * a.ls_conv;
        a.q = reinterpret_cast<Out*>(a.q) + l * a.ls_qk;
        a.k = reinterpret_cast<Out*>(a.k) + l * a.ls_qk;
        a.v = reinterpret_cast<Out*>(a.v) + l * a.ls_v;
        a.beta = reinterpret_cast<Out*>(a.beta) + l * a.ls_tok_h;
        a.gate = reinterpret_cast<Out*>(a.gate) + l * a.ls_tok_h;
    }
    const In* const x = reinterpret_cast<const In*>(a.x);
    const int CG = a.C / 8;   // channel groups per row
    const int K1 = a.K - 1;
    if ((int)blockIdx.x < a.conv_blocks) {
        // ---- short convolution + SiLU (+ L2 normalisation of q and k) over one run of tokens
        const int64_t gi = (int64_t)blockIdx.x * LAYER_THREADS + threadIdx.x;
        const int run = (int)(gi / CG);
        const int ch = (int)(gi % CG) * 8;
        if (run >= a.n_runs) return;   // whole heads leave together: C/8 is a multiple of the lanes of a head
        int lo = 0, hi = a.n_req;      // request of the run: last r with run_cu[r] <= run
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (a.run_cu[mid] <= run) lo = mid; else hi = mid;
        }
        const int r = lo;
        const int t_first = (run - a.run_cu[r]) * LAYER_RUN;          // local index of the run's first token
        const int64_t row0 = a.cu[r];
        const int n = min(LAYER_RUN, a.cu[r + 1] - a.cu[r] - t_first);
        // taps as four weights per channel, older taps of a shorter convolution are zero
        float w4[8][4], bias[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            if (a.K == 4) {
                const float4 t = reinterpret_cast<const float4*>(a.w)[ch + c];
                w4[c][0] = t.x; w4[c][1] = t.y; w4[c][2] = t.z; w4[c][3] = t.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int jj = j - (4 - a.K);
                    w4[c][j] = jj >= 0 ? a.w[(int64_t)(ch + c) * a.K + jj] : 0.f;
                }
            }
            bias[c] = a.bias ? a.bias[ch + c] : 0.f;
        }
        // the three inputs before the run: from the sequence, else from the stored state, else zero
        F8 win[3];
        const int slot = a.src_slot[r];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int s = t_first - 3 + i;
            const int srow = K1 + s;   // row of the stored state when s < 0
            if (s >= 0) {
                win[i] = load8(x + (row0 + s) * a.C + ch);
            } else if (slot >= 0 && srow >= 0) {
                win[i] = load8(reinterpret_cast<const In*>(a.conv_src) + slot * a.src_stride + (int64_t)srow * a.C + ch);
            } else {
                win[i] = F8{{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}};
            }
        }
        // section of the channels: q and k rows are [H_qk d_k] wide, v rows [H_v d_v]
        const bool is_v = ch >= 2 * a.nq;
        const int base = ch < a.nq ? 0 : (is_v ? 2 * a.nq : a.nq);
        const int width = is_v ? a.C - 2 * a.nq : a.nq;
        Out* const dst = reinterpret_cast<Out*>(ch < a.nq ? a.q : (is_v ? a.v : a.k)) + (ch - base);
        const In* src = x + (row0 + t_first) * a.C + ch;
        // four rows at a time; the next four are fetched (raw) while these are worked on
        decltype(load_raw8(src)) nxt[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) nxt[u] = load_raw8(src + (int64_t)min(u, n - 1) * a.C);
        for (int t0 = 0; t0 < n; t0 += 4) {
            decltype(load_raw8(src)) cur[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
            if (t0 + 4 < n) {
#pragma unroll
                for (int u = 0; u < 4; ++u) nxt[u] = load_raw8(src + (int64_t)min(t0 + 4 + u, n - 1) * a.C);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (t0 + u >= n) break;   // uniform over the lanes of a head (same run)
                const F8 xc = widen8(cur[u]);
                F8 y;
                float ss = 0.f;
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    float acc = bias[c];
                    acc = fmaf(w4[c][0], win[0].f[c], acc);
                    acc = fmaf(w4[c][1], win[1].f[c], acc);
                    acc = fmaf(w4[c][2], win[2].f[c], acc);
                    acc = fmaf(w4[c][3], xc.f[c], acc);
                    y.f[c] = silu_f(acc);
                    ss = fmaf(y.f[c], y.f[c], ss);
                }
                win[0] = win[1];
                win[1] = win[2];
                win[2] = xc;
                if (!is_v) {   // uniform over the lanes of a head
                    const float inv = rsqrtf(head_sum(ss, a.d_k) + a.qk_eps);
#pragma unroll
                    for (int c = 0; c < 8; ++c) y.f[c] *= inv;
                }
                store8(dst + (row0 + t_first + t0 + u) * width, y);
            }
        }
        return;
    }
    if ((int)blockIdx.x < a.conv_blocks + a.gate_blocks) {
        // ---- beta = sigmoid(b_pre), gate = exp(-exp(A_log) softplus(a_pre + dt_bias))
        const int64_t e = (int64_t)(blockIdx.x - a.conv_blocks) * LAYER_THREADS + threadIdx.x;
        if (e >= a.T * a.H_v) return;
        const int h = (int)(e % a.H_v);
        const float bp = load1(reinterpret_cast<const In*>(a.b_pre) + e);
        const float ap = load1(reinterpret_cast<const In*>(a.a_pre) + e) + a.dt_bias[h];
        const float sp = fmaxf(ap, 0.f) + log1pf(__expf(-fabsf(ap)));
        store1(reinterpret_cast<Out*>(a.beta) + e, __builtin_amdgcn_rcpf(1.f + __expf(-bp)));
        store1(reinterpret_cast<Out*>(a.gate) + e, __expf(-__expf(a.A_log[h]) * sp));
        return;
    }
    {
        // ---- convolution state at an emit position: the K-1 inputs up to it, oldest first
        const int64_t gi = (int64_t)(blockIdx.x - a.conv_blocks - a.gate_blocks) * LAYER_THREADS + threadIdx.x;
        const int ch = (int)(gi % CG) * 8;
        const int64_t rowi = gi / CG;
        const int j = (int)(rowi % K1);
        const int64_t e = rowi / K1;
        if (e >= a.n_emit) return;
        const int r = a.emit_req[e];
        const int consumed = a.emit_pos[e] - a.start[r];   // tokens of the request up to the position
        const int s = consumed - K1 + j;
        const int slot = a.src_slot[r];
        In* const out = reinterpret_cast<In*>(a.conv_dst) + a.emit_slot[e] * a.dst_stride + (int64_t)j * a.C + ch;
        uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
        const In* from = nullptr;
        if (s >= 0) from = x + ((int64_t)a.cu[r] + s) * a.C + ch;
        else if (slot >= 0 && K1 + s >= 0)
            from = reinterpret_cast<const In*>(a.conv_src) + slot * a.src_stride + (int64_t)(K1 + s) * a.C + ch;
        if (from) {
            v0 = reinterpret_cast<const uint4*>(from)[0];
            if (sizeof(In) == 4) v1 = reinterpret_cast<const uint4*>(from)[1];
        }
        reinterpret_cast<uint4*>(out)[0] = v0;
        if (sizeof(In) == 4) reinterpret_cast<uint4*>(out)[1] = v1;
    }
}

struct LayerOutArgs {
    const void* o;       // [T][H_v][d_v]
    const void* z;       // [T][H_v][d_v]
    const float* weight; // [d_v]
    void* y;
    int64_t n_groups;    // T * H_v * d_v / 8
    int64_t ls_tok;      // stacked layers (grid.y): elements from one layer's plane of o, z, y to the next
    int32_t d_v;
    float eps;
};

// y = o / sqrt(mean(o^2) + eps) * weight * SiLU(z) per (token, head); a thread owns 8 adjacent channels.
template <typename O, typename In, typename Out>
__global__ void __launch_bounds__(LAYER_THREADS) gdn_layer_output_kernel(LayerOutArgs a) {
    const int64_t gi = (int64_t)blockIdx.x * LAYER_THREADS + threadIdx.x;
    if (gi >= a.n_groups) return;   // whole heads leave together
    const int c0 = (int)(gi % (a.d_v / 8)) * 8;
    const int64_t lo = (int64_t)blockIdx.y * a.ls_tok;   // this block's layer
    const F8 o = load8_once(reinterpret_cast<const O*>(a.o) + lo + gi * 8);   // o and z are not read again
    const F8 z = load8_once(reinterpret_cast<const In*>(a.z) + lo + gi * 8);
    const F8 w = load8(a.weight + (int64_t)blockIdx.y * a.d_v + c0);
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) ss = fmaf(o.f[c], o.f[c], ss);
    ss = head_sum(ss, a.d_v);
    const float inv = rsqrtf(ss / (float)a.d_v + a.eps);
    F8 y;
#pragma unroll
    for (int c = 0; c < 8; ++c) y.f[c] = o.f[c] * inv * w.f[c] * silu_f(z.f[c]);
    store8(reinterpret_cast<Out*>(a.y) + lo + gi * 8, y);
}

}  // namespace gdn
