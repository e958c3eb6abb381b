"""ctypes front end of the C oracle (oracle/gdn_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's CPU-baseline leg may import this module.
It imports nothing from the HIP package and the HIP package imports nothing from here.

The arithmetic lives in the C file; this module only marshals numpy arrays.  The two
checkpoint-pool copies (gather, scatter) are the definition written out with numpy
indexing: Sec. 6 (overhead decomposition) names loading a stored checkpoint as a step
of a cache hit, and Sec. 3 fixes what a checkpoint is (the exact state at position c).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gdn_oracle.c")
_LIB = os.path.join(_HERE, "libgdn_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (CPU code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
             "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_deepest_ckpt.restype = ctypes.c_int
        lib.oracle_deepest_ckpt.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int32]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_resume_prefill.restype = ctypes.c_int
        lib.oracle_resume_prefill.argtypes = (
            [ctypes.c_int] * 5 + [ctypes.c_double, ctypes.c_int, ctypes.c_int64]
            + [ctypes.c_void_p] * 5 + [ctypes.c_int] + [ctypes.c_void_p] * 3 + [ctypes.c_int]
            + [ctypes.c_void_p] * 5)
        _lib = lib
    return _lib


def _i32(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None and a.size else ctypes.c_void_p(0)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def deepest_ckpt(pos, t: int) -> int:
    """Sec. 3: index of max{c in C : c <= t}, or -1 for the zero state at position 0."""
    pos = _i32(pos)
    return int(_load().oracle_deepest_ckpt(_ptr(pos), int(pos.size), int(t)))


def resume_prefill(q, k, v, beta, gate, cu_seqlens, start_pos, src_slot, emit_cu, emit_pos,
                   state_src=None, scale: float = 1.0):
    """Run the token loop.

    q, k: [L][T][H_qk][d_k]; v: [L][T][H_v][d_v]; beta, gate: [L][T][H_v]; all float32, or
    all uint16 holding bf16 bits.  state_src: float32 (the pool's type) or float64
    [n_slots][L][H_v][d_v][d_k], or None.
    Returns (o float64 [L][T][H_v][d_v], states float64 [n_emit][L][H_v][d_v][d_k]).
    """
    lib = _load()
    arrs = [np.ascontiguousarray(x) for x in (q, k, v, beta, gate)]
    dt = arrs[0].dtype
    if any(a.dtype != dt for a in arrs):
        raise ValueError("q, k, v, beta, gate must share one dtype")
    if dt == np.float32:
        code = F32
    elif dt == np.uint16:
        code = BF16
    else:
        raise ValueError("inputs must be float32 or uint16 (bf16 bits)")
    q, k, v, beta, gate = arrs
    L, T, H_qk, d_k = q.shape
    H_v, d_v = v.shape[2], v.shape[3]
    assert k.shape == q.shape and v.shape[:2] == (L, T)
    assert beta.shape == (L, T, H_v) and gate.shape == (L, T, H_v)
    cu, sp, ss = _i32(cu_seqlens), _i32(start_pos), _i32(src_slot)
    ecu, epos = _i32(emit_cu), _i32(emit_pos)
    n_req = sp.size
    assert cu.size == n_req + 1 and ss.size == n_req and ecu.size == n_req + 1
    assert int(cu[-1]) <= T and int(ecu[-1]) == epos.size
    if state_src is not None:
        state_src = np.ascontiguousarray(state_src)
        assert state_src.dtype in (np.float32, np.float64)
        assert state_src.shape[1:] == (L, H_v, d_v, d_k)
        assert ss.max(initial=-1) < state_src.shape[0]
    else:
        assert ss.max(initial=-1) < 0, "a source slot needs state_src"
    n_emit = epos.size
    o = np.zeros((L, T, H_v, d_v), dtype=np.float64)
    states = np.zeros((n_emit, L, H_v, d_v, d_k), dtype=np.float64)
    rc = lib.oracle_resume_prefill(L, H_qk, H_v, d_k, d_v, float(scale), code, T,
                                   _ptr(q), _ptr(k), _ptr(v), _ptr(beta), _ptr(gate),
                                   n_req, _ptr(cu), _ptr(sp), _ptr(state_src),
                                   int(state_src is not None and state_src.dtype == np.float64), _ptr(ss),
                                   _ptr(ecu), _ptr(epos), _ptr(states), _ptr(o))
    if rc != 0:
        raise RuntimeError(f"oracle_resume_prefill failed: {rc}")
    return o, states


def ckpt_gather(pool, slot_ids):
    """dst[i] = pool[slot_ids[i]], zeros for slot id -1 (position 0: the zero state)."""
    pool = np.asarray(pool)
    ids = np.asarray(slot_ids, dtype=np.int64)
    out = np.zeros((ids.size,) + pool.shape[1:], dtype=pool.dtype)
    for i, s in enumerate(ids):
        if s >= 0:
            out[i] = pool[s]
    return out


def ckpt_scatter(pool, slot_ids, src):
    """pool[slot_ids[i]] = src[i]; returns the updated copy of the pool."""
    out = np.array(pool, copy=True)
    for i, s in enumerate(np.asarray(slot_ids, dtype=np.int64)):
        out[s] = src[i]
    return out
