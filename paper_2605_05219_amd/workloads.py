"""Seeded synthetic inputs for the resume-prefill path.  Serves the oracle tests and the GPU
tests alike and holds none of the method's arithmetic: it draws token streams, checkpoint
positions, overlap depths and slot ids, and lays requests out in the packed form both sides
consume.  The one method-defined quantity it needs, the deepest reusable checkpoint
l(t;C) of Sec. 3, is passed in by the caller as a function, so each side uses its own.

The streams stand in for GatedDeltaNet activations of the model the paper measures and the
depth laws for the overlap-depth distributions of its datasets (Sec. 5, "Datasets" and
"Overlap distributions"): neither the weights nor the datasets are available, only their
shapes are imitated (near-full-length spike, concentrated non-uniform overlap, log-spread
suffix lengths).

numpy only; bf16 is carried as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

import numpy as np

DeepestFn = Callable[[Sequence[int], int], int]


# ----------------------------------------------------------------------------- dtypes
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 values -> the array handed to either side ('f32': float32, 'bf16': uint16 bits)."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def to_f32(x: np.ndarray) -> np.ndarray:
    """Storage array -> the exact fp32 values it encodes."""
    return bf16_bits_to_f32(x) if x.dtype == np.uint16 else np.asarray(x, dtype=np.float32)


# ----------------------------------------------------------------------------- streams
@dataclass
class Streams:
    """Per-token inputs of one sequence for all layers and heads (storage dtype)."""
    q: np.ndarray      # [L][T][H_qk][d_k]
    k: np.ndarray      # [L][T][H_qk][d_k]
    v: np.ndarray      # [L][T][H_v][d_v]
    beta: np.ndarray   # [L][T][H_v]
    gate: np.ndarray   # [L][T][H_v]

    @property
    def T(self) -> int:
        return self.q.shape[1]

    def fields(self):
        return (self.q, self.k, self.v, self.beta, self.gate)

    def slice(self, lo: int, hi: int) -> "Streams":
        return Streams(*(a[:, lo:hi] for a in self.fields()))


def concat_streams(parts: Sequence[Streams]) -> Streams:
    return Streams(*(np.ascontiguousarray(np.concatenate([p.fields()[i] for p in parts], axis=1))
                     for i in range(5)))


def token_streams(rng: np.random.Generator, L: int, T: int, H_qk: int, H_v: int, d_k: int,
                  d_v: int, dtype: str, gate_mode: str = "config") -> Streams:
    """The configs' recipe: q, k ~ N(0,1) L2-normalised per head (in fp32, then rounded);
    v ~ N(0,1); beta = sigmoid(N(0,1)); gate a = exp(-softplus(N(0,1))).

    gate_mode: 'config' as above; 'slow' raises a to the power 1/16 so that a state
    survives thousands of tokens; 'one' sets a = 1 (ungated delta rule).
    """
    def normal(*shape):
        return rng.standard_normal(shape, dtype=np.float32)

    q = normal(L, T, H_qk, d_k)
    k = normal(L, T, H_qk, d_k)
    q /= np.linalg.norm(q, axis=-1, keepdims=True)
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = normal(L, T, H_v, d_v)
    beta = 1.0 / (1.0 + np.exp(-normal(L, T, H_v)))
    z = normal(L, T, H_v)
    softplus = np.log1p(np.exp(-np.abs(z))) + np.maximum(z, 0.0)
    if gate_mode == "config":
        gate = np.exp(-softplus)
    elif gate_mode == "slow":
        gate = np.exp(-softplus / 16.0)
    elif gate_mode == "one":
        gate = np.ones_like(z)
    else:
        raise ValueError(gate_mode)
    return Streams(*(to_storage(a.astype(np.float32), dtype) for a in (q, k, v, beta, gate)))


# ----------------------------------------------------------------------------- positions
def balanced_positions(N: int, M: int) -> List[int]:
    """Table 1, 'Balanced': floor(i (N+1) / (M+1)), i = 1..M."""
    return [(i * (N + 1)) // (M + 1) for i in range(1, M + 1)]


def uniform_aligned_positions(N: int, M: int) -> List[int]:
    """i N / M, i = 1..M: evenly spaced, block aligned when N/M is, and N itself included."""
    return [(i * N) // M for i in range(1, M + 1)]


def snap_positions(raw: Sequence[int], N: int, M: int, block: int = 128) -> List[int]:
    """Clip drawn positions to block boundaries (Sec. 5: every checkpoint position is clipped
    to a block boundary), drop 0 and duplicates, then refill to M with the nearest free
    multiples of `block` so that the budget is used."""
    got = sorted({min(N - N % block, max(block, int(round(p / block)) * block)) for p in raw})
    free = [m for m in range(block, N + 1, block) if m not in got]
    for p in sorted(raw):
        if len(got) >= M or not free:
            break
        nearest = min(free, key=lambda m: abs(m - p))
        free.remove(nearest)
        got.append(nearest)
    return sorted(got)[:M] if len(got) > M else sorted(got)


# ----------------------------------------------------------------------------- packed calls
@dataclass
class Call:
    """Host-side arguments of one resume-prefill call, in the layout both sides share."""
    L: int
    H_qk: int
    H_v: int
    d_k: int
    d_v: int
    dtype: str                     # 'f32' or 'bf16'
    streams: Streams               # packed over requests: [L][T_total]...
    cu_seqlens: np.ndarray         # int32 [n_req+1]
    start_pos: np.ndarray          # int32 [n_req]  absolute position of the loaded state
    src_slot: np.ndarray           # int32 [n_req]  pool slot of that state, -1 = zero state
    emit_cu: np.ndarray            # int32 [n_req+1]
    emit_pos: np.ndarray           # int32 [n_emit] absolute positions, increasing per request
    emit_slot: np.ndarray          # int32 [n_emit] destination pool slots
    n_slots: int
    meta: dict = field(default_factory=dict)

    @property
    def n_req(self) -> int:
        return int(self.start_pos.size)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def slot_shape(self):
        return (self.L, self.H_v, self.d_v, self.d_k)


def pack_call(L, H_qk, H_v, d_k, d_v, dtype, per_request: Sequence[Streams], start_pos, src_slot,
              emit_lists: Sequence[Sequence[int]], emit_slots: Sequence[Sequence[int]],
              n_slots: int, meta: Optional[dict] = None) -> Call:
    lens = [s.T for s in per_request]
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    ecu = np.zeros(len(lens) + 1, dtype=np.int32)
    ecu[1:] = np.cumsum([len(e) for e in emit_lists])
    flat = lambda ll: np.asarray([x for l in ll for x in l], dtype=np.int32)
    if per_request:
        streams = concat_streams(per_request)
    else:
        z = lambda *s: np.zeros(s, dtype=np.float32 if dtype == "f32" else np.uint16)
        streams = Streams(z(L, 0, H_qk, d_k), z(L, 0, H_qk, d_k), z(L, 0, H_v, d_v),
                          z(L, 0, H_v), z(L, 0, H_v))
    return Call(L, H_qk, H_v, d_k, d_v, dtype, streams, cu,
                np.asarray(start_pos, dtype=np.int32), np.asarray(src_slot, dtype=np.int32),
                ecu, flat(emit_lists), flat(emit_slots), n_slots, dict(meta or {}))


def full_prefill_call(prefix: Streams, positions: Sequence[int], slots: Sequence[int],
                      n_slots: int, dtype: str) -> Call:
    """One request that runs the whole prefix from the zero state and stores the state at
    every checkpoint position (building the cache entry)."""
    L, _, H_qk, d_k = prefix.q.shape
    H_v, d_v = prefix.v.shape[2], prefix.v.shape[3]
    return pack_call(L, H_qk, H_v, d_k, d_v, dtype, [prefix], [0], [-1], [list(positions)],
                     [list(slots)], n_slots, {"kind": "full", "positions": list(positions)})


def resume_call(prefix: Streams, positions: Sequence[int], slots: Sequence[int],
                depths: Sequence[int], ends: Sequence[int], tails: Sequence[Optional[Streams]],
                deepest: DeepestFn, first_free_slot: int, n_slots: int, dtype: str,
                emit_rule: Callable[[int, int], List[int]]) -> Call:
    """Requests that overlap the cached prefix up to depth t_r.

    Request r resumes from the deepest checkpoint l_r at or below t_r (Sec. 3), replays the
    shared tokens l_r+1 .. min(t_r, end) copied from the prefix, then its own tail.  Its own
    tokens are `tails[r]`; when the request ends inside the prefix (`ends[r] <= N` and no
    tail), the tokens after t_r are still the prefix's.  emit_rule(l, end) lists the
    absolute positions whose states the request stores; they go to fresh slots counted up
    from first_free_slot.
    """
    L, N, H_qk, d_k = prefix.q.shape
    H_v, d_v = prefix.v.shape[2], prefix.v.shape[3]
    per_req, start, src, elists, eslots = [], [], [], [], []
    nxt = first_free_slot
    for t, end, tail in zip(depths, ends, tails):
        i = deepest(positions, int(t))
        l = int(positions[i]) if i >= 0 else 0
        parts = []
        shared_hi = min(int(t), int(end)) if tail is not None else int(end)
        if shared_hi > l:
            parts.append(prefix.slice(l, shared_hi))
        if tail is not None and tail.T > 0:
            parts.append(tail)
        if parts:
            s = concat_streams(parts)
        else:
            s = prefix.slice(0, 0)
        assert s.T == int(end) - l, (s.T, end, l)
        per_req.append(s)
        start.append(l)
        src.append(int(slots[i]) if i >= 0 else -1)
        e = emit_rule(l, int(end))
        elists.append(e)
        eslots.append(list(range(nxt, nxt + len(e))))
        nxt += len(e)
    assert nxt <= n_slots, "pool too small for the fresh slots"
    return pack_call(L, H_qk, H_v, d_k, d_v, dtype, per_req, start, src, elists, eslots, n_slots,
                     {"kind": "resume", "positions": list(map(int, positions)),
                      "depths": list(map(int, depths)), "ends": list(map(int, ends))})


def emit_downstream(positions: Sequence[int]) -> Callable[[int, int], List[int]]:
    """Store every checkpoint position inside (l, end], plus end itself."""
    def rule(l: int, end: int) -> List[int]:
        e = sorted({int(c) for c in positions if l < c <= end} | ({end} if end > l else set()))
        return e
    return rule


def emit_every(step: int) -> Callable[[int, int], List[int]]:
    """Store every multiple of `step` inside (l, end], plus end itself."""
    def rule(l: int, end: int) -> List[int]:
        e = sorted(set(range((l // step + 1) * step, end + 1, step)) | ({end} if end > l else set()))
        return e
    return rule


# ----------------------------------------------------------------------------- depth laws
def depths_uniform(rng, n: int, N: int) -> np.ndarray:
    """Config 1: depth uniform over [0, N)."""
    return rng.integers(0, N, size=n)


def depths_mixture(rng, n: int, N: int, lo: int) -> np.ndarray:
    """Config 2: half of the mass uniform over [lo, N], the rest uniform over [1, N]."""
    pick = rng.random(n) < 0.5
    return np.where(pick, rng.integers(lo, N + 1, size=n), rng.integers(1, N + 1, size=n))


def depths_truncated_geometric(rng, n: int, N: int, mean_frac: float = 0.8) -> np.ndarray:
    """Config 3: mass piled at the full length, t = N - min(G, N-1), G geometric with mean
    (1 - mean_frac) N, so that the mean depth is about mean_frac N."""
    g = rng.geometric(1.0 / ((1.0 - mean_frac) * N), size=n) - 1
    return N - np.minimum(g, N - 1)


def lengths_log_uniform(rng, n: int, lo: int, hi: int) -> np.ndarray:
    """Config 4: suffix lengths log-uniform in [lo, hi]."""
    return np.clip(np.round(np.exp(rng.uniform(np.log(lo), np.log(hi), size=n))), lo, hi).astype(np.int64)


# ----------------------------------------------------------------------------- the configs
@dataclass
class Scenario:
    """A cached prefix entry plus the resume call against it."""
    name: str
    prefix: Streams
    positions: List[int]
    slots: List[int]
    build: Call            # full prefill that fills the checkpoint slots
    resume: Call
    n_slots: int


def _scenario(name, rng, L, H_qk, H_v, d, N, positions, depths, ends, tail_len, dtype, deepest,
              gate_mode="config", emit_rule=None) -> Scenario:
    prefix = token_streams(rng, L, N, H_qk, H_v, d, d, dtype, gate_mode)
    slots = list(range(len(positions)))
    n_req = len(depths)
    tails = []
    for t, end in zip(depths, ends):
        n_tail = tail_len(int(t), int(end))
        tails.append(token_streams(rng, L, n_tail, H_qk, H_v, d, d, dtype, gate_mode)
                     if n_tail is not None else None)
    rule = emit_rule or emit_downstream(positions)
    # upper bound on fresh slots: every request may emit at most len(positions)+1 states
    n_emit_max = sum(len(rule(0, int(e))) for e in ends)
    n_slots = len(positions) + n_emit_max
    build = full_prefill_call(prefix, positions, slots, n_slots, dtype)
    resume = resume_call(prefix, positions, slots, depths, ends, tails, deepest, len(positions),
                         n_slots, dtype, rule)
    resume.meta["config"] = name
    return Scenario(name, prefix, list(positions), slots, build, resume, n_slots)


def config0(deepest: DeepestFn, seed: int = 1000, dtype: str = "f32", gate_mode="config") -> Scenario:
    """1 layer, 2 heads, d=64, N=512, checkpoints {128,256,384}, resume from 256 to 512."""
    rng = np.random.default_rng(seed)
    N = 512
    return _scenario("config0", rng, 1, 2, 2, 64, N, [128, 256, 384], [256], [N],
                     lambda t, e: None, dtype, deepest, gate_mode)


def config1(deepest: DeepestFn, seed: int = 1001, n_draws: int = 1, N: int = 8192, M: int = 16,
            H: int = 16, d: int = 128, dtype: str = "bf16", gate_mode="config",
            positions: Optional[Sequence[int]] = None) -> Scenario:
    """1 layer, 16 heads, d=128, N=8192, M=16 uniformly spaced checkpoints; depth uniform over
    [0,N).  Each draw is a batch-1 request: tokens up to the depth are the prefix's, the rest
    are its own, it runs to N and stores every downstream checkpoint state."""
    rng = np.random.default_rng(seed)
    pos = list(positions) if positions is not None else uniform_aligned_positions(N, M)
    depths = depths_uniform(rng, n_draws, N)
    return _scenario("config1", rng, 1, H, H, d, N, pos, depths, [N] * n_draws,
                     lambda t, e: e - t, dtype, deepest, gate_mode)


def config2(deepest: DeepestFn, seed: int = 1002, n_req: int = 64, N: int = 16384, M: int = 12,
            H: int = 16, d: int = 128, tail: int = 256, dtype: str = "bf16",
            gate_mode="config") -> Scenario:
    """Batched resume against one shared entry, M non-uniform positions (a third drawn in
    the first 73% of the prefix, the rest in the last 27%, where half of the depth mass
    lies), varlen suffixes plus a fresh tail per request."""
    rng = np.random.default_rng(seed)
    lo = (N * 12000) // 16384
    n_early = M // 3
    raw = list(rng.integers(1, lo, size=n_early)) + list(rng.integers(lo, N + 1, size=M - n_early))
    pos = snap_positions(raw, N, M)
    depths = depths_mixture(rng, n_req, N, lo)
    ends = [int(t) + tail for t in depths]
    return _scenario("config2", rng, 1, H, H, d, N, pos, depths, ends,
                     lambda t, e: e - t, dtype, deepest, gate_mode)


def config3(deepest: DeepestFn, seed: int = 1003, n_req: int = 32, N: int = 32768, M: int = 8,
            H_qk: int = 16, H_v: int = 32, d: int = 128, dtype: str = "bf16",
            gate_mode="config") -> Scenario:
    """Long document, grouped value heads (two per query/key head), M positions in the last
    40% of the prefix, depths piled at the full length; a request ends at its depth."""
    rng = np.random.default_rng(seed)
    raw = list(rng.integers(int(0.6 * N), N + 1, size=M))
    pos = snap_positions(raw, N, M)
    depths = depths_truncated_geometric(rng, n_req, N)
    return _scenario("config3", rng, 1, H_qk, H_v, d, N, pos, depths, [int(t) for t in depths],
                     lambda t, e: None, dtype, deepest, gate_mode)


def config4_call(seed: int = 1004, n_req: int = 256, L: int = 8, H: int = 16, d: int = 128,
                 n_slots: int = 4096, lo: int = 64, hi: int = 8192, emit_step: int = 1024,
                 dtype: str = "bf16", gate_mode="config") -> Call:
    """Layer-group serving step: each request gathers its start state by slot id, replays a
    suffix of log-uniform length and stores states at every multiple of emit_step inside the
    suffix plus its end, to freshly assigned slots.  Layers are independent problems with
    their own streams (no weights exist to chain them).  Start positions are multiples of
    128 (block-clipped checkpoints).  The start states themselves are the caller's to fill.
    """
    rng = np.random.default_rng(seed)
    lens = lengths_log_uniform(rng, n_req, lo, hi)
    starts = rng.integers(1, 64, size=n_req) * 128
    ids = rng.permutation(n_slots)
    src = ids[:n_req]
    rule = emit_every(emit_step)
    per_req, elists, eslots = [], [], []
    nxt = n_req
    for r in range(n_req):
        per_req.append(token_streams(rng, L, int(lens[r]), H, H, d, d, dtype, gate_mode))
        e = rule(int(starts[r]), int(starts[r] + lens[r]))
        elists.append(e)
        eslots.append([int(x) for x in ids[nxt:nxt + len(e)]])
        nxt += len(e)
    assert nxt <= n_slots, "pool too small"
    return pack_call(L, H, H, d, d, dtype, per_req, starts, src, elists, eslots, n_slots,
                     {"kind": "serving", "config": "config4", "lens": [int(x) for x in lens]})


# ----------------------------------------------------------------------------- layer front/back end inputs
@dataclass
class LayerCase:
    """Seeded inputs of the layer's elementwise front and back ends for a packed batch of resumed
    requests (storage dtype for activations and convolution states, fp32 parameters).  Draws only:
    pre-activations ~ N(0,1), taps ~ N(0, 0.5^2), small biases, A_log ~ U(log 0.5, log 4),
    dt_bias ~ N(0, 0.5^2), norm weight 1 + 0.1 N(0,1); they stand in for the projections of the
    model the paper measures (Sec. 6, prototype wall-clock time), whose weights are not available."""
    H_qk: int
    H_v: int
    d_k: int
    d_v: int
    K: int
    dtype: str
    x_qkv: np.ndarray        # [T][C]
    conv_w: np.ndarray       # fp32 [C][K]
    conv_b: np.ndarray       # fp32 [C]
    a_pre: np.ndarray        # [T][H_v]
    b_pre: np.ndarray
    A_log: np.ndarray        # fp32 [H_v]
    dt_bias: np.ndarray
    z: np.ndarray            # [T][H_v][d_v]
    o: np.ndarray            # fp32 [T][H_v][d_v]: stands in for the recurrence output
    norm_w: np.ndarray       # fp32 [d_v]
    conv_pool: np.ndarray    # [n_slots][K-1][C]: stored convolution states (random rows: any rows are legal inputs)
    cu_seqlens: np.ndarray
    start_pos: np.ndarray
    src_slot: np.ndarray
    emit_cu: np.ndarray
    emit_pos: np.ndarray
    emit_slot: np.ndarray

    @property
    def C(self) -> int:
        return 2 * self.H_qk * self.d_k + self.H_v * self.d_v

    @property
    def T(self) -> int:
        return int(self.cu_seqlens[-1])


def layer_case(seed: int, H_qk: int, H_v: int, d_k: int, d_v: int, K: int, dtype: str, lens: Sequence[int],
               starts: Sequence[int], emits: Sequence[Sequence[int]], n_src_slots: int = 4) -> LayerCase:
    """lens[r] tokens from position starts[r]; starts[r] == 0 resumes from nothing (slot -1), otherwise from a
    random source slot; emits[r] are absolute positions in (starts[r], starts[r] + lens[r]]; destination slots
    are fresh ids after the source slots."""
    rng = np.random.default_rng(seed)
    C = 2 * H_qk * d_k + H_v * d_v
    T = int(sum(lens))

    def normal(*shape, s=1.0):
        return (rng.standard_normal(shape, dtype=np.float32) * np.float32(s)).astype(np.float32)

    cu = np.zeros(len(lens) + 1, np.int32)
    cu[1:] = np.cumsum(lens)
    ecu = np.zeros(len(lens) + 1, np.int32)
    ecu[1:] = np.cumsum([len(e) for e in emits])
    epos = np.asarray([p for e in emits for p in e], np.int32)
    src = np.asarray([-1 if s == 0 else int(rng.integers(0, n_src_slots)) for s in starts], np.int32)
    eslot = (n_src_slots + rng.permutation(max(int(epos.size), 1))[:epos.size]).astype(np.int32)
    return LayerCase(
        H_qk, H_v, d_k, d_v, K, dtype,
        to_storage(normal(T, C), dtype), normal(C, K, s=0.5), normal(C, s=0.1),
        to_storage(normal(T, H_v), dtype), to_storage(normal(T, H_v), dtype),
        rng.uniform(np.log(0.5), np.log(4.0), H_v).astype(np.float32), normal(H_v, s=0.5),
        to_storage(normal(T, H_v, d_v), dtype), normal(T, H_v, d_v), (1.0 + normal(d_v, s=0.1)).astype(np.float32),
        to_storage(normal(n_src_slots + max(int(epos.size), 1), K - 1, C), dtype),
        cu, np.asarray(starts, np.int32), src, ecu, epos, eslot)


# ----------------------------------------------------------------------------- attention side of a hit
@dataclass
class AttnCase:
    """Seeded inputs of the attention layers' side of a cache hit for a packed batch of resumed
    requests, all bf16 bit patterns.  Draws only: queries, keys, values (and the output gate's
    pre-activation) ~ N(0,1) times a chosen spread; they stand in for the projections of the model
    the paper measures (Sec. 6, prototype wall-clock time), whose weights are not available.  Request r
    owns sequence slot seq_slot[r]; k_full[r] / v_full[r] hold its keys and values of positions
    1 .. start+len (the restored prefix, then the suffix)."""
    H_q: int
    H_kv: int
    d: int
    q: np.ndarray                 # [T][H_q][d]
    gate: np.ndarray              # [T][H_q][d]
    k_full: List[np.ndarray]      # per request [start+len][H_kv][d]
    v_full: List[np.ndarray]
    cu_seqlens: np.ndarray
    start_pos: np.ndarray
    seq_slot: np.ndarray
    n_slots: int
    cap: int

    @property
    def T(self) -> int:
        return int(self.cu_seqlens[-1])

    def suffix(self, which: str) -> np.ndarray:
        """Packed [T][H_kv][d] keys ('k') or values ('v') of the suffix tokens."""
        full = self.k_full if which == "k" else self.v_full
        parts = [f[s:] for f, s in zip(full, self.start_pos)]
        return np.concatenate(parts, axis=0) if parts else np.zeros((0, self.H_kv, self.d), np.uint16)


def attn_case(seed: int, H_q: int, H_kv: int, d: int, lens: Sequence[int], starts: Sequence[int],
              cap: Optional[int] = None, q_spread: float = 1.0, spare_slots: int = 1) -> AttnCase:
    rng = np.random.default_rng(seed)
    T = int(sum(lens))
    n_req = len(lens)

    def normal(*shape, s=1.0):
        return f32_to_bf16_bits((rng.standard_normal(shape, dtype=np.float32) * np.float32(s)).astype(np.float32))

    cu = np.zeros(n_req + 1, np.int32)
    cu[1:] = np.cumsum(lens)
    need = max([int(s) + int(l) for s, l in zip(starts, lens)] + [1])
    cap = int(cap if cap is not None else need)
    assert cap >= need
    n_slots = n_req + spare_slots
    slot = rng.permutation(n_slots)[:n_req].astype(np.int32)
    q = normal(T, H_q, d, s=q_spread)
    gate = normal(T, H_q, d)
    k_full = [normal(int(s) + int(l), H_kv, d) for s, l in zip(starts, lens)]
    v_full = [normal(int(s) + int(l), H_kv, d) for s, l in zip(starts, lens)]
    return AttnCase(H_q, H_kv, d, q, gate, k_full, v_full, cu, np.asarray(starts, np.int32), slot, n_slots, cap)
