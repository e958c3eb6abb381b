"""Oracle of the attention layers' side of a cache hit.  TEST INFRASTRUCTURE ONLY.

Only tests/ and the smoke entry point may import this module.  Plain numpy, fp64, the definition per head with
a library matmul as the only primitive; it shares no code with the library.

The paper's hybrid runs keep the full attention KV cache next to the sparse recurrent checkpoints
(Table 1, caption) and name the load of the attention layers' cached keys and values as the third
part of a cache hit's cost (Sec. 6, overhead decomposition); its timed layer group holds one full
attention layer (Sec. 6, prototype wall-clock time).  The paper does not restate attention.  What is
computed is causal softmax attention of the recomputed suffix over the restored prefix:

  a request resumed at position c (keys and values 1..c restored from the cache) with suffix
  tokens c+1 .. c+n computes, for suffix token t and query head h,

      o_t[h] = sum_{j=1..t} softmax_j(scale * q_t[h] . k_j[g]) v_j[g],      g = h // (H_q / H_kv)

  (grouped-query attention: consecutive query heads share a key/value head), the keys and values
  c+1..t being the suffix's own, which are also appended to the cache.

Optional output gate (gated attention as in the Qwen3-Next family): y = o * sigmoid(gate).
"""
from __future__ import annotations

import numpy as np


def append_kv(k_cache, v_cache, k_new, v_new, start: int):
    """Rows start .. start+n-1 (0-based) of one request's cache [cap][H_kv][d] take the suffix's
    keys and values; everything else is left as it is.  Returns new arrays."""
    k_cache = np.array(k_cache, copy=True)
    v_cache = np.array(v_cache, copy=True)
    n = k_new.shape[0]
    assert start >= 0 and start + n <= k_cache.shape[0]
    k_cache[start:start + n] = k_new
    v_cache[start:start + n] = v_new
    return k_cache, v_cache


def attention_suffix(q, k_all, v_all, start: int, scale: float):
    """q: [n][H_q][d] queries of suffix tokens start+1 .. start+n (1-based positions);
    k_all, v_all: [start+n][H_kv][d] keys and values of positions 1 .. start+n.
    Returns o [n][H_q][d] in fp64."""
    q = np.asarray(q, dtype=np.float64)
    k_all = np.asarray(k_all, dtype=np.float64)
    v_all = np.asarray(v_all, dtype=np.float64)
    n, H_q, d = q.shape
    total, H_kv, _ = k_all.shape
    assert total == start + n and H_q % H_kv == 0
    group = H_q // H_kv
    o = np.zeros((n, H_q, v_all.shape[2]), dtype=np.float64)
    pos_q = start + 1 + np.arange(n)            # 1-based position of each query
    pos_k = 1 + np.arange(total)                # 1-based position of each key
    visible = pos_k[None, :] <= pos_q[:, None]  # causal: key j is seen by query t iff j <= t
    for h in range(H_q):
        g = h // group
        logits = scale * (q[:, h, :] @ k_all[:, g, :].T)            # [n][total]
        logits = np.where(visible, logits, -np.inf)
        logits = logits - logits.max(axis=1, keepdims=True)         # the softmax is shift-invariant
        w = np.exp(logits)
        w = w / w.sum(axis=1, keepdims=True)
        o[:, h, :] = w @ v_all[:, g, :]
    return o


def output_gate(o, gate):
    """y = o * sigmoid(gate), elementwise."""
    o = np.asarray(o, dtype=np.float64)
    gate = np.asarray(gate, dtype=np.float64)
    return o / (1.0 + np.exp(-gate))
