"""ctypes binding of the checkpoint placement layer (include/ckpt_place.h): argument marshalling only."""
from __future__ import annotations

import ctypes
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .binding import GdnError, lib

_i32, _i64, _vp, _f64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_double

EXPORTS = ["ckpt_place_balanced", "ckpt_place_block", "ckpt_place_sqrt", "ckpt_place_log", "ckpt_clip_to_blocks",
           "ckpt_expected_recompute", "ckpt_place_dp", "ckpt_hist_create", "ckpt_hist_destroy", "ckpt_hist_observe",
           "ckpt_hist_get", "ckpt_hist_solve", "ckpt_online_create", "ckpt_online_destroy", "ckpt_online_observe",
           "ckpt_online_schedule", "ckpt_online_histogram"]

_ready = False


def _lib():
    global _ready
    L = lib()
    if not _ready:
        L.ckpt_place_balanced.restype = _i32
        L.ckpt_place_balanced.argtypes = [_i32, _i32, _vp]
        L.ckpt_place_block.restype = _i32
        L.ckpt_place_block.argtypes = [_i32, _i32, _vp, _i32]
        L.ckpt_place_sqrt.restype = _i32
        L.ckpt_place_sqrt.argtypes = [_i32, _vp, _i32]
        L.ckpt_place_log.restype = _i32
        L.ckpt_place_log.argtypes = [_i32, _i32, _i32, _vp]
        L.ckpt_clip_to_blocks.restype = _i32
        L.ckpt_clip_to_blocks.argtypes = [_vp, _i32, _i32, _vp]
        L.ckpt_expected_recompute.restype = _i32
        L.ckpt_expected_recompute.argtypes = [_vp, _i32, _vp, _i32, _vp, _vp, _vp, _vp]
        L.ckpt_place_dp.restype = _i32
        L.ckpt_place_dp.argtypes = [_vp, _i32, _i32, _vp, _vp]
        L.ckpt_hist_create.restype = _vp
        L.ckpt_hist_create.argtypes = [_i32, _f64]
        L.ckpt_hist_destroy.restype = None
        L.ckpt_hist_destroy.argtypes = [_vp]
        L.ckpt_hist_observe.restype = _i64
        L.ckpt_hist_observe.argtypes = [_vp, _i32]
        L.ckpt_hist_get.restype = _i32
        L.ckpt_hist_get.argtypes = [_vp, _vp]
        L.ckpt_hist_solve.restype = _i32
        L.ckpt_hist_solve.argtypes = [_vp, _i32, _i32, _vp, _vp]
        L.ckpt_online_create.restype = _vp
        L.ckpt_online_create.argtypes = [_i32, _i32, _i32, _f64, _i32]
        L.ckpt_online_destroy.restype = None
        L.ckpt_online_destroy.argtypes = [_vp]
        L.ckpt_online_observe.restype = _i32
        L.ckpt_online_observe.argtypes = [_vp, _i32]
        L.ckpt_online_schedule.restype = _i32
        L.ckpt_online_schedule.argtypes = [_vp, _vp, _i32]
        L.ckpt_online_histogram.restype = _vp
        L.ckpt_online_histogram.argtypes = [_vp]
        _ready = True
    return L


def _count(rc: int, what: str) -> int:
    if rc < 0:
        raise GdnError(rc, what)
    return rc


def _p(p) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(p, dtype=np.float64))


def _pos(pos) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(pos, dtype=np.int32))


def _ptr(a: Optional[np.ndarray]):
    return _vp(a.ctypes.data) if a is not None and a.size else _vp(0)


def ckpt_place_balanced(N: int, M: int) -> List[int]:
    out = np.zeros(max(M, 1), np.int32)
    n = _count(_lib().ckpt_place_balanced(N, M, _ptr(out)), "ckpt_place_balanced")
    return out[:n].tolist()


def ckpt_place_block(N: int, B: int) -> List[int]:
    cap = max(N // max(B, 1), 1)
    out = np.zeros(cap, np.int32)
    n = _count(_lib().ckpt_place_block(N, B, _ptr(out), cap), "ckpt_place_block")
    return out[:n].tolist()


def ckpt_place_sqrt(N: int) -> List[int]:
    cap = max(N, 1)
    out = np.zeros(cap, np.int32)
    n = _count(_lib().ckpt_place_sqrt(N, _ptr(out), cap), "ckpt_place_sqrt")
    return out[:n].tolist()


def ckpt_place_log(N: int, unit: int, M: int) -> List[int]:
    out = np.zeros(max(M, 1), np.int32)
    n = _count(_lib().ckpt_place_log(N, unit, M, _ptr(out)), "ckpt_place_log")
    return out[:n].tolist()


def ckpt_clip_to_blocks(pos: Sequence[int], B: int) -> List[int]:
    a = _pos(pos)
    out = np.zeros(max(a.size, 1), np.int32)
    n = _count(_lib().ckpt_clip_to_blocks(_ptr(a), a.size, B, _ptr(out)), "ckpt_clip_to_blocks")
    return out[:n].tolist()


def ckpt_expected_recompute(p, pos: Sequence[int]) -> Tuple[float, float, float, float]:
    """(E[r], R_nc, Savings, Reduction)."""
    pp, a = _p(p), _pos(pos)
    v = [_f64(0.0) for _ in range(4)]
    _count(_lib().ckpt_expected_recompute(_ptr(pp), pp.size, _ptr(a), a.size, *[ctypes.byref(x) for x in v]),
           "ckpt_expected_recompute")
    return tuple(x.value for x in v)


def ckpt_place_dp(p, M: int) -> Tuple[float, List[int]]:
    """(minimum expected recomputation, one optimal set of at most M positions)."""
    pp = _p(p)
    out = np.zeros(max(M, 1), np.int32)
    cost = _f64(0.0)
    n = _count(_lib().ckpt_place_dp(_ptr(pp), pp.size, M, _ptr(out), ctypes.byref(cost)), "ckpt_place_dp")
    return cost.value, out[:n].tolist()


class OverlapHistogram:
    """Exponentially weighted histogram of observed overlap depths (gamma = 1: plain empirical)."""

    def __init__(self, N: int, gamma: float = 0.99):
        self._h = _lib().ckpt_hist_create(N, gamma)
        if not self._h:
            raise ValueError("ckpt_hist_create: N must be >= 1 and gamma in (0, 1]")
        self.N = N

    def observe(self, t: int) -> int:
        return _count(int(_lib().ckpt_hist_observe(self._h, t)), "ckpt_hist_observe")

    def get(self) -> np.ndarray:
        p = np.zeros(self.N, np.float64)
        _count(_lib().ckpt_hist_get(self._h, _ptr(p)), "ckpt_hist_get")
        return p

    def solve(self, M: int, B: int = 1) -> Tuple[float, List[int]]:
        out = np.zeros(max(M, 1), np.int32)
        cost = _f64(0.0)
        n = _count(_lib().ckpt_hist_solve(self._h, M, B, _ptr(out), ctypes.byref(cost)), "ckpt_hist_solve")
        return cost.value, out[:n].tolist()

    def close(self):
        if self._h:
            _lib().ckpt_hist_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class OnlineScheduler:
    """The online loop: observe overlap depths, re-solve the placement every `period` observations."""

    def __init__(self, N: int, M: int, B: int = 1, gamma: float = 0.99, period: int = 10):
        self._o = _lib().ckpt_online_create(N, M, B, gamma, period)
        if not self._o:
            raise ValueError("ckpt_online_create: N, M, B, period must be >= 1 and gamma in (0, 1]")
        self.N, self.M = N, M

    def observe(self, t: int) -> bool:
        return bool(_count(int(_lib().ckpt_online_observe(self._o, t)), "ckpt_online_observe"))

    def schedule(self) -> List[int]:
        out = np.zeros(self.M, np.int32)
        n = _count(_lib().ckpt_online_schedule(self._o, _ptr(out), self.M), "ckpt_online_schedule")
        return out[:n].tolist()

    def histogram(self) -> np.ndarray:
        p = np.zeros(self.N, np.float64)
        _count(_lib().ckpt_hist_get(_lib().ckpt_online_histogram(self._o), _ptr(p)), "ckpt_hist_get")
        return p

    def close(self):
        if self._o:
            _lib().ckpt_online_destroy(self._o)
            self._o = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
