"""ctypes binding of the layer front and back ends (include/gdn_layer.h): argument marshalling only."""
from __future__ import annotations

import ctypes

from .binding import GDN_BF16, GDN_F32, _check, _dp, _h32, _hp, _stream_ptr, lib

_i32, _i64, _vp, _f32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_float

EXPORTS = ["gdn_layer_workspace_bytes", "gdn_layer_inputs", "gdn_layer_output"]


class gdn_layer_shape(ctypes.Structure):
    _fields_ = [("H_qk", _i32), ("H_v", _i32), ("d_k", _i32), ("d_v", _i32), ("conv_k", _i32), ("in_dtype", _i32),
                ("out_dtype", _i32), ("o_dtype", _i32), ("qk_eps", _f32), ("norm_eps", _f32), ("L", _i32), ("T_alloc", _i64)]


def make_layer_shape(H_qk, H_v, d_k, d_v, conv_k=4, in_dtype="bf16", out_dtype="bf16", o_dtype="f32", qk_eps=1e-6,
                     norm_eps=1e-5, L=1, T_alloc=0) -> gdn_layer_shape:
    code = {"f32": GDN_F32, "bf16": GDN_BF16, GDN_F32: GDN_F32, GDN_BF16: GDN_BF16}
    return gdn_layer_shape(H_qk, H_v, d_k, d_v, conv_k, code[in_dtype], code[out_dtype], code[o_dtype], float(qk_eps),
                           float(norm_eps), int(L), int(T_alloc))


_ready = False


def _lib():
    global _ready
    L = lib()
    if not _ready:
        L.gdn_layer_workspace_bytes.restype = _i64
        L.gdn_layer_workspace_bytes.argtypes = [_i32, _i32]
        L.gdn_layer_inputs.restype = _i32
        L.gdn_layer_inputs.argtypes = ([ctypes.POINTER(gdn_layer_shape)] + [_vp] * 7 + [_i32, _vp, _vp] + [_vp, _i64, _i32, _vp]
                                       + [_vp, _vp] + [_vp, _i64, _i32, _vp] + [_vp] * 5 + [_vp, _i64, _vp])
        L.gdn_layer_output.restype = _i32
        L.gdn_layer_output.argtypes = [ctypes.POINTER(gdn_layer_shape), _vp, _vp, _vp, _vp, _i64, _vp]
        _ready = True
    return L


def gdn_layer_workspace_bytes(n_req: int, n_emit: int) -> int:
    return _check(int(_lib().gdn_layer_workspace_bytes(int(n_req), int(n_emit))), "gdn_layer_workspace_bytes")


def gdn_layer_inputs(shape: gdn_layer_shape, x_qkv, conv_w, conv_b, a_pre, b_pre, A_log, dt_bias, cu_seqlens, start_pos,
                     conv_src, src_slot, emit_cu, emit_pos, conv_dst, emit_slot, q, k, v, beta, gate, workspace,
                     stream=None) -> None:
    """See include/gdn_layer.h.  Device arguments are torch tensors (or None), index arrays are host sequences;
    pools are [n_slots][K-1][C] tensors whose first stride is the slot stride."""
    cu, sp, ss = _h32(cu_seqlens), _h32(start_pos), _h32(src_slot)
    ecu, epos, eslot = _h32(emit_cu), _h32(emit_pos), _h32(emit_slot)
    _check(_lib().gdn_layer_inputs(
        ctypes.byref(shape), _dp(x_qkv), _dp(conv_w), _dp(conv_b), _dp(a_pre), _dp(b_pre), _dp(A_log), _dp(dt_bias),
        int(sp.size), _hp(cu), _hp(sp),
        _dp(conv_src), int(conv_src.stride(0)) if conv_src is not None else 0,
        int(conv_src.shape[0]) if conv_src is not None else 0, _hp(ss),
        _hp(ecu), _hp(epos),
        _dp(conv_dst), int(conv_dst.stride(0)) if conv_dst is not None else 0,
        int(conv_dst.shape[0]) if conv_dst is not None else 0, _hp(eslot),
        _dp(q), _dp(k), _dp(v), _dp(beta), _dp(gate),
        _dp(workspace), int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream_ptr(stream)), "gdn_layer_inputs")


def gdn_layer_output(shape: gdn_layer_shape, o, z, weight, y, T: int, stream=None) -> None:
    """See include/gdn_layer.h: y = RMS-normalised o times weight times SiLU(z)."""
    _check(_lib().gdn_layer_output(ctypes.byref(shape), _dp(o), _dp(z), _dp(weight), _dp(y), int(T), _stream_ptr(stream)),
           "gdn_layer_output")
