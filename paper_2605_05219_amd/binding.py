"""Thin ctypes binding of the C ABI in include/gdn_resume.h: argument marshalling only.

Device buffers are torch tensors (torch is used for device memory and streams, nothing
else); index arrays are host numpy int32.  Every step of the path runs inside the library.
The library must be present: there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgdn_resume.so")

GDN_F32, GDN_BF16 = 0, 1
GDN_CHUNK = 64

ERRORS = {
    -1: "GDN_ERR_NULL", -2: "GDN_ERR_ALIGN", -3: "GDN_ERR_SHAPE", -4: "GDN_ERR_SEQLENS",
    -5: "GDN_ERR_SLOT_RANGE", -6: "GDN_ERR_SLOT_DUP", -7: "GDN_ERR_SLOT_HAZARD", -8: "GDN_ERR_EMIT",
    -9: "GDN_ERR_WORKSPACE", -10: "GDN_ERR_START", -11: "GDN_ERR_COUNT", -12: "GDN_ERR_STATIC_LIMIT",
}


class GdnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = int(code)
        name = ERRORS.get(self.code, f"GDN_ERR_HIP(hipError {-1000 - self.code})" if self.code <= -1000 else "?")
        super().__init__(f"{where} failed: {self.code} {name}")


class gdn_shape(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int32), ("H_qk", ctypes.c_int32), ("H_v", ctypes.c_int32),
                ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32), ("in_dtype", ctypes.c_int32),
                ("o_dtype", ctypes.c_int32), ("scale", ctypes.c_float), ("T_alloc", ctypes.c_int64)]


_lib = None
_vp, _i32, _i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64


def lib():
    """The loaded library; raises when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2605_05219_amd.build)")
        # PyTorch ships its own HIP runtime; it must be in the process before this library is loaded so
        # that both resolve to the same one (device pointers of one runtime mean nothing to another).
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        L.gdn_version.restype = _i32
        L.gdn_tune_slab_rounds.restype = _i32
        L.gdn_tune_slab_rounds.argtypes = [_i32]
        L.gdn_tune_fused.restype = _i32
        L.gdn_tune_fused.argtypes = [_i32]
        L.gdn_tune_fused_pair.restype = _i32
        L.gdn_tune_fused_pair.argtypes = [_i32]
        L.gdn_tune_fused_per_cu.restype = _i32
        L.gdn_tune_fused_per_cu.argtypes = [_i32]
        L.gdn_profile_enable.restype = _i32
        L.gdn_profile_enable.argtypes = [_i32]
        L.gdn_profile_collect.restype = _i32
        L.gdn_profile_collect.argtypes = [_vp, _vp, _vp, _vp, _vp]
        L.gdn_probe_ceilings.restype = _i32
        L.gdn_probe_ceilings.argtypes = [_vp, _i64, _vp, _vp, _vp]
        L.gdn_deepest_ckpt.restype = _i32
        L.gdn_deepest_ckpt.argtypes = [_vp, _i32, _i32]
        L.gdn_plan_chunks.restype = _i32
        L.gdn_plan_chunks.argtypes = [_i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32]
        L.gdn_workspace_bytes.restype = _i64
        L.gdn_workspace_bytes.argtypes = [ctypes.POINTER(gdn_shape), _i32, _i64, _i32]
        L.gdn_workspace_bytes_fused.restype = _i64
        L.gdn_workspace_bytes_fused.argtypes = [ctypes.POINTER(gdn_shape), _i32, _i64, _i32]
        L.ckpt_gather.restype = _i32
        L.ckpt_gather.argtypes = [_vp, _i64, _i32, _vp, _i32, _vp, _i64, _i64, _vp]
        L.ckpt_scatter.restype = _i32
        L.ckpt_scatter.argtypes = [_vp, _i64, _i32, _vp, _i32, _vp, _i64, _i64, _vp]
        L.gdn_resume_prefill_host.restype = _i32
        L.gdn_resume_prefill_host.argtypes = ([ctypes.POINTER(gdn_shape)] + [_vp] * 5 + [_i32, _vp, _vp]
                                              + [_vp, _i64, _i32, _vp, _vp, _vp] + [_vp, _i64, _i32, _vp] + [_vp, _vp, _i64, _vp])
        L.gdn_workspace_bytes_host.restype = _i64
        L.gdn_workspace_bytes_host.argtypes = [ctypes.POINTER(gdn_shape), _i32, _i64, _i32]
        for f in (L.ckpt_fetch_host, L.ckpt_spill_host):
            f.restype = _i32
            f.argtypes = [_vp, _i64, _i32, _vp, _vp, _i64, _i32, _vp, _i32, _i64, _vp]
        L.gdn_decode_step.restype = _i32
        L.gdn_decode_step.argtypes = [ctypes.POINTER(gdn_shape)] + [_vp] * 5 + [_i32, _vp, _i64, _i32, _vp, _vp, _vp]
        L.gdn_resume_prefill.restype = _i32
        L.gdn_resume_prefill.argtypes = ([ctypes.POINTER(gdn_shape)] + [_vp] * 5 + [_i32, _vp, _vp]
                                         + [_vp, _i64, _i32, _vp] + [_vp, _vp]
                                         + [_vp, _i64, _i32, _vp] + [_vp, _vp, _i64, _vp])
        L.gdn_resume_prefill_static.restype = _i32
        L.gdn_resume_prefill_static.argtypes = ([ctypes.POINTER(gdn_shape)] + [_vp] * 5 + [_i32, _vp, _vp]
                                                + [_vp, _i64, _i32, _vp] + [_vp, _vp]
                                                + [_vp, _i64, _i32, _vp] + [_vp, _vp])
        L.gdn_static_plan_capacity.restype = _i64
        _lib = L
    return _lib


EXPORTS = ["gdn_version", "gdn_tune_slab_rounds", "gdn_tune_fused", "gdn_tune_fused_pair", "gdn_tune_fused_per_cu", "gdn_profile_enable", "gdn_profile_collect", "gdn_probe_ceilings", "gdn_deepest_ckpt", "gdn_plan_chunks", "gdn_workspace_bytes",
           "gdn_workspace_bytes_fused",
           "ckpt_gather", "ckpt_scatter", "gdn_resume_prefill", "gdn_decode_step", "ckpt_fetch_host", "ckpt_spill_host",
           "gdn_workspace_bytes_host", "gdn_resume_prefill_host", "gdn_resume_prefill_static", "gdn_static_plan_capacity"]


def _h32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _hp(a: Optional[np.ndarray]):
    return _vp(a.ctypes.data) if a is not None and a.size else _vp(0)


def _dp(t):
    return _vp(t.data_ptr()) if t is not None else _vp(0)


def _stream_ptr(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return _vp(s.cuda_stream)


def _check(rc: int, where: str) -> int:
    if rc < 0:
        raise GdnError(rc, where)
    return rc


def make_shape(L, H_qk, H_v, d_k, d_v, in_dtype, o_dtype, T_alloc, scale=1.0) -> gdn_shape:
    code = {"f32": GDN_F32, "bf16": GDN_BF16, GDN_F32: GDN_F32, GDN_BF16: GDN_BF16}
    return gdn_shape(L, H_qk, H_v, d_k, d_v, code[in_dtype], code[o_dtype], float(scale), int(T_alloc))


# ----------------------------------------------------------------------------- host-only entry points
def gdn_version() -> int:
    return int(lib().gdn_version())


def gdn_tune_slab_rounds(rounds: int) -> int:
    """Fixes the slab length in chunk rounds (<= 0: automatic); returns the previous setting."""
    return int(lib().gdn_tune_slab_rounds(int(rounds)))


def gdn_tune_fused(mode: int) -> int:
    """1: always the fused kernel where it applies, 0: never, < 0: automatic; returns the previous setting."""
    return int(lib().gdn_tune_fused(int(mode)))


def gdn_tune_fused_pair(mode: int) -> int:
    """Fused kernel with grouped value heads: 1: two heads of a query/key head per workgroup wherever the group size is
    even, 0: one head per workgroup, < 0: automatic; returns the previous setting."""
    return int(lib().gdn_tune_fused_pair(int(mode)))


def gdn_tune_fused_per_cu(n: int) -> int:
    """Workgroups of the fused kernel per compute unit: n >= 1 forces that number (capped at what fits), n < 1: automatic;
    returns the previous setting."""
    return int(lib().gdn_tune_fused_per_cu(int(n)))


def gdn_profile_enable(on: bool) -> None:
    _check(lib().gdn_profile_enable(1 if on else 0), "gdn_profile_enable")


def gdn_profile_collect():
    """(prep kernel ms, recurrence kernel ms, calls, prep launches, recurrence launches) since profiling was enabled."""
    a, b, n = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_int64(0)
    pl, rl = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().gdn_profile_collect(ctypes.byref(a), ctypes.byref(b), ctypes.byref(n), ctypes.byref(pl), ctypes.byref(rl)),
           "gdn_profile_collect")
    return a.value, b.value, n.value, pl.value, rl.value


def gdn_probe_ceilings(scratch, stream=None):
    """(fp16 matrix-instruction TFLOP/s, plain copy GB/s over half of `scratch`) measured on the current device."""
    a, b = ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().gdn_probe_ceilings(_dp(scratch), int(scratch.numel() * scratch.element_size()), ctypes.byref(a), ctypes.byref(b),
                                    _stream_ptr(stream)), "gdn_probe_ceilings")
    return a.value, b.value


def gdn_deepest_ckpt(pos: Sequence[int], t: int) -> int:
    p = _h32(pos)
    return int(lib().gdn_deepest_ckpt(_hp(p), int(p.size), int(t)))


def gdn_plan_chunks(cu_seqlens, start_pos, emit_cu, emit_pos, capacity: Optional[int] = None):
    cu, sp, ecu, epos = _h32(cu_seqlens), _h32(start_pos), _h32(emit_cu), _h32(emit_pos)
    n_req = int(sp.size)
    if capacity is None:
        capacity = int(cu[-1]) // GDN_CHUNK + n_req + int(epos.size) + 1 if cu.size else 1
    tok0 = np.zeros(max(capacity, 1), np.int32)
    ln = np.zeros_like(tok0)
    em = np.zeros_like(tok0)
    rcu = np.zeros(n_req + 1, np.int32)
    nc = _check(lib().gdn_plan_chunks(n_req, _hp(cu), _hp(sp), _hp(ecu), _hp(epos), _hp(tok0), _hp(ln),
                                      _hp(em), _vp(rcu.ctypes.data), int(capacity)), "gdn_plan_chunks")
    return tok0[:nc].copy(), ln[:nc].copy(), em[:nc].copy(), rcu


def gdn_workspace_bytes(shape: gdn_shape, n_req: int, total_tokens: int, n_emit: int) -> int:
    return _check(lib().gdn_workspace_bytes(ctypes.byref(shape), int(n_req), int(total_tokens), int(n_emit)),
                  "gdn_workspace_bytes")


def gdn_workspace_bytes_fused(shape: gdn_shape, n_req: int, total_tokens: int, n_emit: int) -> int:
    """The plan-only workspace that makes a call run the fused kernel (see include/gdn_resume.h)."""
    return _check(lib().gdn_workspace_bytes_fused(ctypes.byref(shape), int(n_req), int(total_tokens), int(n_emit)),
                  "gdn_workspace_bytes_fused")


# ----------------------------------------------------------------------------- device entry points
def ckpt_gather(pool, slot_ids, dst, state_elems: Optional[int] = None, stream=None) -> None:
    """dst[i] = pool[slot_ids[i]] (zeros for -1).  pool: [n_slots, ...] fp32, dst: [n, ...] fp32."""
    ids = _h32(slot_ids)
    n_slots, sstride = int(pool.shape[0]), int(pool.stride(0))
    dstride = int(dst.stride(0)) if dst.dim() > 0 and dst.shape[0] > 0 else sstride
    elems = int(state_elems if state_elems is not None else pool[0].numel())
    _check(lib().ckpt_gather(_dp(pool), sstride, n_slots, _hp(ids), int(ids.size), _dp(dst), dstride, elems,
                             _stream_ptr(stream)), "ckpt_gather")


def ckpt_scatter(pool, slot_ids, src, state_elems: Optional[int] = None, stream=None) -> None:
    """pool[slot_ids[i]] = src[i]."""
    ids = _h32(slot_ids)
    n_slots, sstride = int(pool.shape[0]), int(pool.stride(0))
    srcstride = int(src.stride(0)) if src.dim() > 0 and src.shape[0] > 0 else sstride
    elems = int(state_elems if state_elems is not None else pool[0].numel())
    _check(lib().ckpt_scatter(_dp(pool), sstride, n_slots, _hp(ids), int(ids.size), _dp(src), srcstride, elems,
                              _stream_ptr(stream)), "ckpt_scatter")


def gdn_resume_prefill(shape: gdn_shape, q, k, v, beta, gate, cu_seqlens, start_pos,
                       state_src, src_slot, emit_cu, emit_pos, state_dst, emit_slot,
                       o, workspace, stream=None) -> None:
    """See include/gdn_resume.h.  q..gate, o, state pools and workspace are device tensors;
    the index arrays are host sequences."""
    cu, sp, ss = _h32(cu_seqlens), _h32(start_pos), _h32(src_slot)
    ecu, epos, eslot = _h32(emit_cu), _h32(emit_pos), _h32(emit_slot)
    n_req = int(sp.size)
    if cu.size != n_req + 1 or ecu.size != n_req + 1 or ss.size != n_req or eslot.size != epos.size:
        raise ValueError("index arrays have inconsistent lengths")
    src_stride = int(state_src.stride(0)) if state_src is not None else 0
    src_n = int(state_src.shape[0]) if state_src is not None else 0
    dst_stride = int(state_dst.stride(0)) if state_dst is not None else 0
    dst_n = int(state_dst.shape[0]) if state_dst is not None else 0
    ws_bytes = int(workspace.numel() * workspace.element_size()) if workspace is not None else 0
    _check(lib().gdn_resume_prefill(ctypes.byref(shape), _dp(q), _dp(k), _dp(v), _dp(beta), _dp(gate),
                                    n_req, _hp(cu), _hp(sp),
                                    _dp(state_src), src_stride, src_n, _hp(ss), _hp(ecu), _hp(epos),
                                    _dp(state_dst), dst_stride, dst_n, _hp(eslot),
                                    _dp(o), _dp(workspace), ws_bytes, _stream_ptr(stream)),
           "gdn_resume_prefill")


def gdn_resume_prefill_static(shape: gdn_shape, q, k, v, beta, gate, cu_seqlens, start_pos,
                              state_src, src_slot, emit_cu, emit_pos, state_dst, emit_slot, o, stream=None) -> None:
    """gdn_resume_prefill without a workspace: the plan lives in the library's static device array and nothing is
    allocated (see include/gdn_resume.h)."""
    cu, sp, ss = _h32(cu_seqlens), _h32(start_pos), _h32(src_slot)
    ecu, epos, eslot = _h32(emit_cu), _h32(emit_pos), _h32(emit_slot)
    n_req = int(sp.size)
    if cu.size != n_req + 1 or ecu.size != n_req + 1 or ss.size != n_req or eslot.size != epos.size:
        raise ValueError("index arrays have inconsistent lengths")
    src_stride = int(state_src.stride(0)) if state_src is not None else 0
    src_n = int(state_src.shape[0]) if state_src is not None else 0
    dst_stride = int(state_dst.stride(0)) if state_dst is not None else 0
    dst_n = int(state_dst.shape[0]) if state_dst is not None else 0
    _check(lib().gdn_resume_prefill_static(ctypes.byref(shape), _dp(q), _dp(k), _dp(v), _dp(beta), _dp(gate),
                                           n_req, _hp(cu), _hp(sp),
                                           _dp(state_src), src_stride, src_n, _hp(ss), _hp(ecu), _hp(epos),
                                           _dp(state_dst), dst_stride, dst_n, _hp(eslot),
                                           _dp(o), _stream_ptr(stream)),
           "gdn_resume_prefill_static")


def gdn_static_plan_capacity() -> int:
    return int(lib().gdn_static_plan_capacity())


def gdn_decode_step(shape: gdn_shape, q, k, v, beta, gate, pool, slot, o, stream=None) -> None:
    """See include/gdn_resume.h: one token per request, states updated in place in their pool slots."""
    sl = _h32(slot)
    n_req = int(sl.size)
    _check(lib().gdn_decode_step(ctypes.byref(shape), _dp(q), _dp(k), _dp(v), _dp(beta), _dp(gate), n_req,
                                 _dp(pool), int(pool.stride(0)) if pool is not None else 0,
                                 int(pool.shape[0]) if pool is not None else 0, _hp(sl), _dp(o), _stream_ptr(stream)),
           "gdn_decode_step")


def gdn_workspace_bytes_host(shape: gdn_shape, n_req: int, total_tokens: int, n_emit: int) -> int:
    return _check(int(lib().gdn_workspace_bytes_host(ctypes.byref(shape), n_req, total_tokens, n_emit)),
                  "gdn_workspace_bytes_host")


def _tier(fn, host_pool, host_ids, dev_pool, dev_ids, state_elems, stream):
    hi, di = _h32(host_ids), _h32(dev_ids)
    if hi.size != di.size:
        raise ValueError("host_ids and dev_ids differ in length")
    elems = int(state_elems if state_elems is not None else host_pool[0].numel())
    _check(getattr(lib(), fn)(_dp(host_pool), int(host_pool.stride(0)), int(host_pool.shape[0]), _hp(hi),
                              _dp(dev_pool), int(dev_pool.stride(0)), int(dev_pool.shape[0]), _hp(di), int(hi.size),
                              elems, _stream_ptr(stream)), fn)


def ckpt_fetch_host(host_pool, host_ids, dev_pool, dev_ids, state_elems=None, stream=None) -> None:
    """dev_pool[dev_ids[i]] = host_pool[host_ids[i]] (host_pool: pinned host tensor)."""
    _tier("ckpt_fetch_host", host_pool, host_ids, dev_pool, dev_ids, state_elems, stream)


def ckpt_spill_host(host_pool, host_ids, dev_pool, dev_ids, state_elems=None, stream=None) -> None:
    """host_pool[host_ids[i]] = dev_pool[dev_ids[i]]."""
    _tier("ckpt_spill_host", host_pool, host_ids, dev_pool, dev_ids, state_elems, stream)


def gdn_resume_prefill_host(shape: gdn_shape, q, k, v, beta, gate, cu_seqlens, start_pos,
                            host_state_src, src_slot, emit_cu, emit_pos, state_dst, emit_slot,
                            o, workspace, stream=None) -> None:
    """gdn_resume_prefill with the start states in a pinned host pool (see include/gdn_resume.h)."""
    cu, sp, ss = _h32(cu_seqlens), _h32(start_pos), _h32(src_slot)
    ecu, epos, eslot = _h32(emit_cu), _h32(emit_pos), _h32(emit_slot)
    n_req = int(sp.size)
    if cu.size != n_req + 1 or ecu.size != n_req + 1 or ss.size != n_req or eslot.size != epos.size:
        raise ValueError("index arrays have inconsistent lengths")
    src_stride = int(host_state_src.stride(0)) if host_state_src is not None else 0
    src_n = int(host_state_src.shape[0]) if host_state_src is not None else 0
    dst_stride = int(state_dst.stride(0)) if state_dst is not None else 0
    dst_n = int(state_dst.shape[0]) if state_dst is not None else 0
    ws_bytes = int(workspace.numel() * workspace.element_size()) if workspace is not None else 0
    _check(lib().gdn_resume_prefill_host(ctypes.byref(shape), _dp(q), _dp(k), _dp(v), _dp(beta), _dp(gate),
                                         n_req, _hp(cu), _hp(sp),
                                         _dp(host_state_src), src_stride, src_n, _hp(ss), _hp(ecu), _hp(epos),
                                         _dp(state_dst), dst_stride, dst_n, _hp(eslot),
                                         _dp(o), _dp(workspace), ws_bytes, _stream_ptr(stream)),
           "gdn_resume_prefill_host")
