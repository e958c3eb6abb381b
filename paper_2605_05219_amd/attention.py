"""ctypes binding of the attention layers' side of a cache hit (include/attn_resume.h): argument marshalling only."""
from __future__ import annotations

import ctypes

from .binding import GDN_BF16, GDN_F32, _check, _dp, _h32, _hp, _stream_ptr, lib

_i32, _i64, _vp, _f32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_float

EXPORTS = ["attn_workspace_bytes", "attn_kv_restore", "attn_kv_spill", "attn_suffix_prefill", "attn_plan", "attn_tune_split",
           "attn_tune_pack"]


class attn_shape(ctypes.Structure):
    _fields_ = [("H_q", _i32), ("H_kv", _i32), ("d", _i32), ("o_dtype", _i32), ("scale", _f32)]


def make_attn_shape(H_q, H_kv, d, o_dtype="f32", scale=None) -> attn_shape:
    code = {"f32": GDN_F32, "bf16": GDN_BF16, GDN_F32: GDN_F32, GDN_BF16: GDN_BF16}
    return attn_shape(H_q, H_kv, d, code[o_dtype], float(d ** -0.5 if scale is None else scale))


_ready = False


def _lib():
    global _ready
    L = lib()
    if not _ready:
        L.attn_workspace_bytes.restype = _i64
        L.attn_workspace_bytes.argtypes = [ctypes.POINTER(attn_shape), _i32, _i64]
        L.attn_kv_restore.restype = _i32
        L.attn_kv_restore.argtypes = ([ctypes.POINTER(attn_shape), _i32, _vp] + [_vp, _vp, _i64, _i32, _vp]
                                      + [_vp, _vp, _i64, _i32, _i32, _vp] + [_vp])
        L.attn_kv_spill.restype = _i32
        L.attn_kv_spill.argtypes = L.attn_kv_restore.argtypes
        L.attn_suffix_prefill.restype = _i32
        L.attn_suffix_prefill.argtypes = ([ctypes.POINTER(attn_shape)] + [_vp] * 4 + [_i32, _vp, _vp]
                                          + [_vp, _vp, _i64, _i32, _i32, _vp] + [_vp, _vp, _i64, _vp])
        L.attn_plan.restype = _i32
        L.attn_plan.argtypes = [ctypes.POINTER(attn_shape), _i32, _vp, _vp, _i32] + [_vp] * 8
        for f in (L.attn_tune_split, L.attn_tune_pack):
            f.restype = _i32
            f.argtypes = [_i32]
        _ready = True
    return L


def attn_tune_split(allow: bool) -> bool:
    """False: key walks are never cut into parts; True: automatic.  Returns the previous setting."""
    return bool(_lib().attn_tune_split(1 if allow else 0))


def attn_tune_pack(allow: bool) -> bool:
    """False: one query head per workgroup always; True: automatic.  Returns the previous setting."""
    return bool(_lib().attn_tune_pack(1 if allow else 0))


def attn_workspace_bytes(shape: attn_shape, n_req: int, total_tokens: int) -> int:
    return _check(int(_lib().attn_workspace_bytes(ctypes.byref(shape), int(n_req), int(total_tokens))), "attn_workspace_bytes")


def attn_plan(shape: attn_shape, cu_seqlens, start_pos, capacity: int = 1 << 16):
    """See include/attn_resume.h: (units as an int32 array [n_units][5] of (req, tile, t0, t1, part), heads per row
    group, key tile rows).  Host only."""
    import numpy as np
    cu, sp = _h32(cu_seqlens), _h32(start_pos)
    arrs = [np.zeros(capacity, np.int32) for _ in range(5)]
    n, pack, kt = _i32(0), _i32(0), _i32(0)
    _check(_lib().attn_plan(ctypes.byref(shape), int(sp.size), _hp(cu), _hp(sp), int(capacity), *[_vp(a.ctypes.data) for a in arrs],
                            ctypes.byref(n), ctypes.byref(pack), ctypes.byref(kt)), "attn_plan")
    return np.stack([a[:n.value] for a in arrs], axis=1), pack.value, kt.value


def _pool_geometry(pool):
    """(slot stride in elements, slots, rows per slot) of a [n_slots][cap][H_kv][d] tensor."""
    if pool is None:
        return 0, 0, 0
    return int(pool.stride(0)), int(pool.shape[0]), int(pool.shape[1])


def attn_kv_restore(shape: attn_shape, prefix_len, host_k, host_v, host_slot, k_cache, v_cache, seq_slot, stream=None) -> None:
    """See include/attn_resume.h.  host_k / host_v are host tensors [n_host_slots][cap][H_kv][d] (pinned for
    overlap), k_cache / v_cache device tensors of the same slot geometry; index arrays are host sequences."""
    pl, hs, ss = _h32(prefix_len), _h32(host_slot), _h32(seq_slot)
    stride, n_slots, cap = _pool_geometry(k_cache)
    hstride, hn, _ = _pool_geometry(host_k)
    _check(_lib().attn_kv_restore(ctypes.byref(shape), int(pl.size), _hp(pl), _dp(host_k), _dp(host_v), hstride, hn, _hp(hs),
                                  _dp(k_cache), _dp(v_cache), stride, n_slots, cap, _hp(ss), _stream_ptr(stream)),
           "attn_kv_restore")


def attn_kv_spill(shape: attn_shape, n_rows, host_k, host_v, host_slot, k_cache, v_cache, seq_slot, stream=None) -> None:
    """See include/attn_resume.h: the reverse of attn_kv_restore (device slots to host slots)."""
    nr, hs, ss = _h32(n_rows), _h32(host_slot), _h32(seq_slot)
    stride, n_slots, cap = _pool_geometry(k_cache)
    hstride, hn, _ = _pool_geometry(host_k)
    _check(_lib().attn_kv_spill(ctypes.byref(shape), int(nr.size), _hp(nr), _dp(host_k), _dp(host_v), hstride, hn, _hp(hs),
                                _dp(k_cache), _dp(v_cache), stride, n_slots, cap, _hp(ss), _stream_ptr(stream)),
           "attn_kv_spill")


def attn_suffix_prefill(shape: attn_shape, q, k_new, v_new, out_gate, cu_seqlens, start_pos, k_cache, v_cache, seq_slot, o,
                        workspace, stream=None) -> None:
    """See include/attn_resume.h.  Device arguments are torch tensors (out_gate may be None); the caches are
    [n_slots][cap][H_kv][d] tensors whose first stride is the slot stride; index arrays are host sequences."""
    cu, sp, ss = _h32(cu_seqlens), _h32(start_pos), _h32(seq_slot)
    stride, n_slots, cap = _pool_geometry(k_cache)
    _check(_lib().attn_suffix_prefill(
        ctypes.byref(shape), _dp(q), _dp(k_new), _dp(v_new), _dp(out_gate), int(sp.size), _hp(cu), _hp(sp),
        _dp(k_cache), _dp(v_cache), stride, n_slots, cap, _hp(ss), _dp(o),
        _dp(workspace), int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream_ptr(stream)), "attn_suffix_prefill")
