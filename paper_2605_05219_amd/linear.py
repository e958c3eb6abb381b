"""ctypes binding of the layers' projections (include/gdn_linear.h): argument marshalling only."""
from __future__ import annotations

import ctypes

from .binding import GDN_BF16, GDN_F32, _check, _dp, _stream_ptr, lib

_i32, _i64, _vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p

EXPORTS = ["gdn_linear", "gdn_linear_split", "gdn_linear_tune"]

_ready = False


def _lib():
    global _ready
    L = lib()
    if not _ready:
        L.gdn_linear.restype = _i32
        L.gdn_linear.argtypes = [_vp, _i64, _vp, _i64, _vp, _vp, _i64, _i32, _i64, _i32, _i32, _vp]
        L.gdn_linear_split.restype = _i32
        L.gdn_linear_split.argtypes = [_vp, _i64, _vp, _i64, _vp, _i32, _vp, _vp, _vp, _i32, _i64, _i32, _vp]
        L.gdn_linear_tune.restype = _i32
        L.gdn_linear_tune.argtypes = [_i32]
        _ready = True
    return L


def gdn_linear_raw(x_ptr: int, ldx: int, w_ptr: int, ldw: int, bias_ptr: int, y_ptr: int, ldy: int, out_dtype: int,
                   T: int, N: int, K: int, stream_ptr: int = 0) -> int:
    """The C entry point with plain integers for the pointers; returns the status code (no exception)."""
    return int(_lib().gdn_linear(_vp(x_ptr), int(ldx), _vp(w_ptr), int(ldw), _vp(bias_ptr), _vp(y_ptr), int(ldy),
                                 int(out_dtype), int(T), int(N), int(K), _vp(stream_ptr)))


def gdn_linear(x, w, bias, y, stream=None) -> None:
    """y[t][n] = bias[n] + sum_k x[t][k] w[n][k].  x [T][K] and w [N][K] are bf16 tensors with unit inner stride,
    bias an fp32 [N] tensor or None, y [T][N] bf16 or fp32 with unit inner stride (it may be a column slice of a wider
    tensor: its row stride is passed on)."""
    import torch
    T, K = int(x.shape[0]), int(x.shape[1])
    N = int(w.shape[0])
    if int(w.shape[1]) != K or tuple(y.shape) != (T, N) or (bias is not None and tuple(bias.shape) != (N,)):
        raise ValueError("gdn_linear: shapes do not match")
    if x.dtype != torch.bfloat16 or w.dtype != torch.bfloat16 or (bias is not None and bias.dtype != torch.float32):
        raise ValueError("gdn_linear: x and w are bf16, bias fp32")
    if (K > 1 and (x.stride(1) != 1 or w.stride(1) != 1)) or (N > 1 and y.stride(1) != 1):
        raise ValueError("gdn_linear: inner strides must be 1")
    code = {torch.bfloat16: GDN_BF16, torch.float32: GDN_F32}.get(y.dtype)
    if code is None:
        raise ValueError("gdn_linear: y is bf16 or fp32")
    ldx = int(x.stride(0)) if T > 1 else K
    ldw = int(w.stride(0)) if N > 1 else K
    ldy = int(y.stride(0)) if T > 1 else max(N, int(y.stride(0)))
    _check(_lib().gdn_linear(_dp(x), ldx, _dp(w), ldw, _dp(bias), _dp(y), ldy, code, T, N, K, _stream_ptr(stream)),
           "gdn_linear")


def gdn_linear_tune(shape: int) -> int:
    """Fixes the workgroup tile (0, 1, 2) or returns the choice to the library (-1); returns the previous setting."""
    return int(_lib().gdn_linear_tune(int(shape)))


class SplitPlan:
    """The host arrays of a gdn_linear_split call (column boundaries, destination pointers, leading dimensions), built once
    for calls that repeat."""

    def __init__(self, widths, ptrs, lds):
        n = len(widths)
        if not (len(ptrs) == len(lds) == n):
            raise ValueError("gdn_linear_split: one pointer and one leading dimension per segment")
        cols = [0]
        for wd in widths:
            cols.append(cols[-1] + int(wd))
        self.n_seg = n
        self.N = cols[-1]
        self.cols = (ctypes.c_int32 * (n + 1))(*cols)
        self.ptrs = (ctypes.c_void_p * n)(*[int(p) for p in ptrs])
        self.lds = (ctypes.c_int64 * n)(*[int(v) for v in lds])


def gdn_linear_split_raw(x_ptr: int, ldx: int, w_ptr: int, ldw: int, bias_ptr: int, plan: SplitPlan, out_dtype: int, T: int,
                         K: int, stream_ptr: int = 0) -> int:
    """The C entry point with plain integers for the pointers; returns the status code (no exception)."""
    return int(_lib().gdn_linear_split(_vp(x_ptr), int(ldx), _vp(w_ptr), int(ldw), _vp(bias_ptr), plan.n_seg, plan.cols, plan.ptrs,
                                       plan.lds, int(out_dtype), int(T), int(K), _vp(stream_ptr)))


def gdn_linear_split(x, w, bias, ys, stream=None) -> None:
    """One projection whose outputs go to the tensors `ys` by column range: ys[s] is [T][n_s] (unit inner stride, its row
    stride is passed on), the widths n_s add up to w's rows; all of one dtype (bf16 or fp32)."""
    import torch
    T, K = int(x.shape[0]), int(x.shape[1])
    if int(w.shape[1]) != K or sum(int(y.shape[1]) for y in ys) != int(w.shape[0]) or any(int(y.shape[0]) != T for y in ys):
        raise ValueError("gdn_linear_split: shapes do not match")
    if x.dtype != torch.bfloat16 or w.dtype != torch.bfloat16 or (bias is not None and bias.dtype != torch.float32):
        raise ValueError("gdn_linear_split: x and w are bf16, bias fp32")
    code = {torch.bfloat16: GDN_BF16, torch.float32: GDN_F32}.get(ys[0].dtype)
    if code is None or any(y.dtype != ys[0].dtype for y in ys):
        raise ValueError("gdn_linear_split: the outputs are all bf16 or all fp32")
    if (K > 1 and (x.stride(1) != 1 or w.stride(1) != 1)) or any(int(y.shape[1]) > 1 and y.stride(1) != 1 for y in ys):
        raise ValueError("gdn_linear_split: inner strides must be 1")
    plan = SplitPlan([int(y.shape[1]) for y in ys], [y.data_ptr() for y in ys],
                     [int(y.stride(0)) if T > 1 else max(int(y.shape[1]), int(y.stride(0))) for y in ys])
    ldx = int(x.stride(0)) if T > 1 else K
    ldw = int(w.stride(0)) if int(w.shape[0]) > 1 else K
    _check(gdn_linear_split_raw(x.data_ptr(), ldx, w.data_ptr(), ldw, bias.data_ptr() if bias is not None else 0, plan, code, T, K,
                                _stream_ptr(stream).value or 0), "gdn_linear_split")
