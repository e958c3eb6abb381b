"""Device-side plumbing shared by the tests, `bench.py` and `smoke()`: a packed call's tensors on
the GPU, and the device-generated serving step of configs[4].  Argument marshalling and seeded
draws only; every step of the path runs inside the library.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from . import binding, workloads as wl


def to_device(arr):
    """numpy storage array (uint16 = bf16 bit patterns) -> tensor on the current device."""
    import torch
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(arr).cuda()


class GpuCall:
    """Device copies of a call's tensors plus its output and workspace buffers."""

    def __init__(self, call, pool, o_dtype="f32", scale=1.0, T_alloc=None, dst_pool=None):
        import torch
        self.call = call
        s = call.streams
        T = int(T_alloc if T_alloc is not None else max(call.total_tokens, 1))
        assert T >= call.total_tokens

        def plane(a):
            if a.shape[1] == T:
                return to_device(np.ascontiguousarray(a))
            full = np.zeros((a.shape[0], T) + a.shape[2:], dtype=a.dtype)
            full[:, :a.shape[1]] = a
            return to_device(full)

        self.q, self.k, self.v, self.beta, self.gate = (plane(a) for a in s.fields())
        self.pool = pool if hasattr(pool, "data_ptr") else torch.from_numpy(np.ascontiguousarray(pool)).cuda()
        self.dst_pool = self.pool if dst_pool is None else dst_pool
        self.shape = binding.make_shape(call.L, call.H_qk, call.H_v, call.d_k, call.d_v, call.dtype, o_dtype, T, scale)
        self.o = torch.full((call.L, T, call.H_v, call.d_v), float("nan"),
                            dtype=torch.float32 if o_dtype == "f32" else torch.bfloat16, device="cuda")
        nbytes = binding.gdn_workspace_bytes(self.shape, call.n_req, call.total_tokens, int(call.emit_pos.size))
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")

    def run(self, stream=None):
        c = self.call
        binding.gdn_resume_prefill(self.shape, self.q, self.k, self.v, self.beta, self.gate, c.cu_seqlens,
                                   c.start_pos, self.pool, c.src_slot, c.emit_cu, c.emit_pos, self.dst_pool,
                                   c.emit_slot, self.o, self.workspace, stream)


def run_call_gpu(call, pool, o_dtype="f32", scale=1.0):
    """Returns (o [L][T_total][H_v][d_v] float32, pool after the call as numpy)."""
    import torch
    g = GpuCall(call, pool, o_dtype, scale)
    g.run()
    torch.cuda.synchronize()
    o = g.o[:, :call.total_tokens].float().cpu().numpy()
    return o, g.pool.cpu().numpy()


@dataclass
class ServingStep:
    """configs[4] on the device: 256 requests of log-uniform suffix length through L independent layers of H heads,
    start states gathered by slot id from an n_slots pool, states stored every emit_step positions and at the end
    of each request to fresh slots.  Token tensors and the pool are generated on the device (they are too large
    to generate on the host); index arrays are host numpy."""
    L: int
    H: int
    d: int
    n_slots: int
    lens: np.ndarray
    cu_seqlens: np.ndarray
    start_pos: np.ndarray
    src_slot: np.ndarray
    emit_cu: np.ndarray
    emit_pos: np.ndarray
    emit_slot: np.ndarray
    q: object
    k: object
    v: object
    beta: object
    gate: object
    pool: object
    o: object
    shape: object
    workspace: object
    H_qk: int = 0          # query/key heads when value heads are grouped (0: as many as value heads)

    @property
    def n_req(self) -> int:
        return int(self.lens.size)

    @property
    def T(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def n_emit(self) -> int:
        return int(self.emit_pos.size)

    def run(self, stream=None):
        binding.gdn_resume_prefill(self.shape, self.q, self.k, self.v, self.beta, self.gate, self.cu_seqlens,
                                   self.start_pos, self.pool, self.src_slot, self.emit_cu, self.emit_pos, self.pool,
                                   self.emit_slot, self.o, self.workspace, stream)

    def host_request(self, r: int, layers: List[int]) -> "wl.Call":
        """Request r's tokens of the given layers copied to the host as a one-request call (bf16 bit patterns), with
        its start position, source slot and emit list; slot ids stay those of the device pool."""
        import torch
        lo, hi = int(self.cu_seqlens[r]), int(self.cu_seqlens[r + 1])
        e0, e1 = int(self.emit_cu[r]), int(self.emit_cu[r + 1])
        bits = lambda t: t[layers, lo:hi].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        st = wl.Streams(bits(self.q), bits(self.k), bits(self.v), bits(self.beta), bits(self.gate))
        return wl.pack_call(len(layers), self.H_qk or self.H, self.H, self.d, self.d, "bf16", [st], [int(self.start_pos[r])],
                            [int(self.src_slot[r])], [list(self.emit_pos[e0:e1])], [list(self.emit_slot[e0:e1])],
                            self.n_slots)


def config4_device(seed: int = 1004, n_req: int = 256, L: int = 8, H: int = 16, d: int = 128, n_slots: int = 4096,
                   lo: int = 64, hi: int = 8192, emit_step: int = 1024, o_dtype: str = "f32",
                   pool_scale: float = 0.1, H_qk: int = 0) -> ServingStep:
    """Draws the serving step on the current device.  Recipe of the configs: q, k ~ N(0,1) L2-normalised per head
    (fp32, then rounded to bf16), v ~ N(0,1), beta = sigmoid(N(0,1)), gate = exp(-softplus(N(0,1))); suffix lengths
    log-uniform in [lo, hi]; start positions multiples of 128; pool entries N(0, pool_scale^2) (any state is a valid
    resume point); source slots n_req distinct ids, destination slots fresh distinct ids.  H_qk > 0 gives the H value
    heads H_qk query/key heads to share (grouped value heads)."""
    import torch
    dev = torch.device("cuda")
    rng = np.random.default_rng(seed)
    lens = wl.lengths_log_uniform(rng, n_req, lo, hi)
    starts = (rng.integers(1, 64, size=n_req) * 128).astype(np.int32)
    ids = rng.permutation(n_slots)
    T = int(lens.sum())
    rule = wl.emit_every(emit_step)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    epos, ecu, eslot, nxt = [], [0], [], n_req
    for r in range(n_req):
        e = rule(int(starts[r]), int(starts[r] + lens[r]))
        epos += e
        ecu.append(len(epos))
        eslot += [int(x) for x in ids[nxt:nxt + len(e)]]
        nxt += len(e)
    assert nxt <= n_slots, "pool too small"
    need = n_slots * L * H * d * d * 4 + L * T * H * (3 * d * 2 + d * (4 if o_dtype == "f32" else 2) + 4) + (8 << 30)
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < need:
        raise RuntimeError(f"needs {need >> 30} GiB of device memory, {free_b >> 30} free")
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    rn = lambda *sh: torch.randn(sh, device=dev, generator=g, dtype=torch.float32)
    Hq = H_qk or H
    q = torch.empty((L, T, Hq, d), dtype=torch.bfloat16, device=dev)
    k, v = torch.empty_like(q), torch.empty((L, T, H, d), dtype=torch.bfloat16, device=dev)
    for l in range(L):
        q[l] = torch.nn.functional.normalize(rn(T, Hq, d), dim=-1).bfloat16()
        k[l] = torch.nn.functional.normalize(rn(T, Hq, d), dim=-1).bfloat16()
        v[l] = rn(T, H, d).bfloat16()
    beta = torch.sigmoid(rn(L, T, H)).bfloat16()
    gate = torch.exp(-torch.nn.functional.softplus(rn(L, T, H))).bfloat16()
    pool = torch.empty((n_slots, L, H, d, d), dtype=torch.float32, device=dev)
    step = max(1, min(n_slots, (1 << 30) // (L * H * d * d * 4)))
    for s0 in range(0, n_slots, step):
        n = min(step, n_slots - s0)
        pool[s0:s0 + n] = rn(n, L, H, d, d) * pool_scale
    o = torch.full((L, T, H, d), float("nan"), dtype=torch.float32 if o_dtype == "f32" else torch.bfloat16, device=dev)
    shape = binding.make_shape(L, Hq, H, d, d, "bf16", o_dtype, T)
    # the plan-only workspace: the call runs the fused kernel (the library's own choice for a call of this size)
    ws = torch.empty(max(256, binding.gdn_workspace_bytes_fused(shape, n_req, T, len(epos))), dtype=torch.uint8, device=dev)
    return ServingStep(L, H, d, n_slots, lens, cu, starts, ids[:n_req].astype(np.int32), np.asarray(ecu, np.int32),
                       np.asarray(epos, np.int32), np.asarray(eslot, np.int32), q, k, v, beta, gate, pool, o, shape, ws, Hq)
