"""Oracle of the GatedDeltaNet layer's elementwise front and back ends.  TEST INFRASTRUCTURE ONLY.

Only tests/ may import this module.  Plain numpy, fp64, every function the definition written
out with explicit loops over tokens and taps; it shares no code with the library.

The paper's method applies to layers whose hidden state can be taken out and put back without loss (Sec. 1)
and measures a layer group with GatedDeltaNet layers (Sec. 6, prototype wall-clock time) without
restating the layer.  What is computed here is the published GatedDeltaNet layer around the
recurrence, in the notation of the recurrence oracle (positions 1-based, state "at" position c
= after consuming tokens 1..c):

  short convolution   y_t[c] = SiLU(bias[c] + sum_{j=0..K-1} w[c][j] x_{t-(K-1)+j}[c]), x_s = 0 for s <= 0;
                      depthwise, causal, K taps, tap K-1 on the current token (reading: the
                      cross-correlation convention of the common deep-learning conv1d)
  its state           the last K-1 inputs: rows x_{c-K+2} .. x_c at position c (oldest first); a
                      resumed request continues from the stored rows exactly as if it had seen the
                      whole prefix -- the part of the layer's hidden state that is not the matrix S
  q, k                L2-normalised per head after the convolution: x / sqrt(sum x^2 + eps)
  beta                sigmoid(b_pre)
  gate a              exp(-exp(A_log[h]) * softplus(a_pre + dt_bias[h]))
  output              y = o / sqrt(mean(o^2) + eps) * weight * SiLU(z) per (token, value head)

Channel order of the convolution input: [q heads | k heads | v heads].
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np


def silu(x):
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-x))


def softplus(x):
    x = np.asarray(x, dtype=np.float64)
    return np.log1p(np.exp(-np.abs(x))) + np.maximum(x, 0.0)


def short_conv_pre(x: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray], state: Optional[np.ndarray]) -> np.ndarray:
    """Pre-activation of the short convolution over one sequence.

    x [T][C]; w [C][K]; bias [C] or None; state [K-1][C] (inputs before x[0], oldest first) or None = zeros.
    """
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    T, C = x.shape
    K = w.shape[1]
    y = np.zeros((T, C))
    for t in range(T):
        for j in range(K):
            s = t - (K - 1) + j                 # input row of tap j
            if s >= 0:
                row = x[s]
            elif state is not None:
                row = np.asarray(state[(K - 1) + s], dtype=np.float64)
            else:
                continue
            y[t] += w[:, j] * row
        if bias is not None:
            y[t] += np.asarray(bias, dtype=np.float64)
    return y


def conv_state_after(x: np.ndarray, state: Optional[np.ndarray], K: int, n: int) -> np.ndarray:
    """The K-1 inputs that precede token n (0-based) of a sequence: rows x[n-K+1 .. n-1], taken from
    `state` (or zeros) where they fall before x[0].  n = number of tokens consumed."""
    C = x.shape[1]
    out = np.zeros((K - 1, C))
    for i in range(K - 1):
        s = n - (K - 1) + i
        if s >= 0:
            out[i] = x[s]
        elif state is not None:
            out[i] = state[(K - 1) + s]
    return out


def l2norm(x: np.ndarray, eps: float) -> np.ndarray:
    """x [..., d] -> x / sqrt(sum x^2 + eps) over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt((x * x).sum(axis=-1, keepdims=True) + eps)


def gates(a_pre, b_pre, A_log, dt_bias) -> Tuple[np.ndarray, np.ndarray]:
    """a_pre, b_pre [T][H]; A_log, dt_bias [H] -> (beta, gate)."""
    a_pre = np.asarray(a_pre, dtype=np.float64)
    b_pre = np.asarray(b_pre, dtype=np.float64)
    beta = 1.0 / (1.0 + np.exp(-b_pre))
    g = -np.exp(np.asarray(A_log, dtype=np.float64))[None, :] * softplus(a_pre + np.asarray(dt_bias, dtype=np.float64)[None, :])
    return beta, np.exp(g)


def layer_inputs(x_qkv, conv_w, conv_b, a_pre, b_pre, A_log, dt_bias, H_qk: int, H_v: int, d_k: int, d_v: int,
                 cu_seqlens: Sequence[int], start_pos: Sequence[int], src_slot: Sequence[int], conv_src,
                 emit_cu: Sequence[int], emit_pos: Sequence[int], qk_eps: float):
    """Packed requests -> q [T][H_qk][d_k], k, v [T][H_v][d_v], beta, gate [T][H_v], conv states [n_emit][K-1][C].

    Request r owns rows [cu[r], cu[r+1]) = tokens at positions start_pos[r]+1 ..; its convolution
    continues from conv_src[src_slot[r]] (zeros for slot -1); emit e of request r is the conv state
    at absolute position emit_pos[emit_cu[r] + e].
    """
    x_qkv = np.asarray(x_qkv, dtype=np.float64)
    K = np.asarray(conv_w).shape[1]
    T, C = x_qkv.shape
    nq = H_qk * d_k
    assert C == 2 * nq + H_v * d_v
    q = np.zeros((T, H_qk, d_k))
    k = np.zeros((T, H_qk, d_k))
    v = np.zeros((T, H_v, d_v))
    states: List[np.ndarray] = []
    for r in range(len(start_pos)):
        lo, hi = int(cu_seqlens[r]), int(cu_seqlens[r + 1])
        st = None if int(src_slot[r]) < 0 else np.asarray(conv_src[int(src_slot[r])], dtype=np.float64)
        xs = x_qkv[lo:hi]
        y = silu(short_conv_pre(xs, conv_w, conv_b, st))
        q[lo:hi] = l2norm(y[:, :nq].reshape(-1, H_qk, d_k), qk_eps)
        k[lo:hi] = l2norm(y[:, nq:2 * nq].reshape(-1, H_qk, d_k), qk_eps)
        v[lo:hi] = y[:, 2 * nq:].reshape(-1, H_v, d_v)
        for e in range(int(emit_cu[r]), int(emit_cu[r + 1])):
            states.append(conv_state_after(xs, st, K, int(emit_pos[e]) - int(start_pos[r])))
    beta, gate = gates(a_pre, b_pre, A_log, dt_bias)
    st_out = np.stack(states) if states else np.zeros((0, K - 1, C))
    return q, k, v, beta, gate, st_out


def output_norm_gate(o, z, weight, eps: float) -> np.ndarray:
    """o, z [T][H][d]; weight [d] -> RMS-normalised o times weight times SiLU(z)."""
    o = np.asarray(o, dtype=np.float64)
    ms = (o * o).mean(axis=-1, keepdims=True)
    return o / np.sqrt(ms + eps) * np.asarray(weight, dtype=np.float64) * silu(z)
