"""Oracle of the layer's projections.  TEST INFRASTRUCTURE ONLY: imported by the tests, never by the product path,
and it shares no code with the HIP library.

The paper times a layer group of GatedDeltaNet and attention layers (Sec. 6, prototype wall-clock time) and does not
restate the layers; their projections are the plain affine maps of any such layer,
    y[t][n] = bias[n] + sum_k x[t][k] w[n][k]          (weights stored [out][in]),
written out here as the definition: an explicit triple loop in fp64 for small cases, and the same sum through
numpy's fp64 matrix product for the sizes the parity tests use.  Inputs are the bits the GPU gets (bf16 carried as
uint16, or fp32), widened exactly to fp64.

Pins (tests/test_linear_oracle_pins.py): the two forms against each other, a hand-worked case, the identity and a
permutation matrix, linearity, the bias alone, and the [out][in] storage convention.
"""
from __future__ import annotations

import numpy as np


def _f64(a) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype == np.uint16:                       # bf16 bit patterns
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def linear_loops(x, w, bias=None) -> np.ndarray:
    """The definition, term by term (small inputs only)."""
    x, w = _f64(x), _f64(w)
    T, K = x.shape
    N, K2 = w.shape
    assert K == K2
    b = np.zeros(N) if bias is None else _f64(bias)
    y = np.zeros((T, N), dtype=np.float64)
    for t in range(T):
        for n in range(N):
            acc = b[n]
            for k in range(K):
                acc += x[t, k] * w[n, k]
            y[t, n] = acc
    return y


def linear(x, w, bias=None) -> np.ndarray:
    """The same sum through the fp64 matrix product (rounding order aside)."""
    x, w = _f64(x), _f64(w)
    y = x @ w.T
    if bias is not None:
        y = y + _f64(bias)[None, :]
    return y
