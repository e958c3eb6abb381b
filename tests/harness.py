"""Shared test plumbing: runs one packed call through the oracle or through the HIP library."""
from __future__ import annotations

import numpy as np


def max_norm_err(x, ref) -> float:
    """max |x - ref| / max |ref| over one tensor (the tolerance's 'max rel err')."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    den = np.abs(ref).max()
    return float(np.abs(x - ref).max() / (den if den > 0 else 1.0))


def run_call_oracle(call, pool):
    from oracle import gdn_oracle as orc
    s = call.streams
    return orc.resume_prefill(s.q, s.k, s.v, s.beta, s.gate, call.cu_seqlens, call.start_pos, call.src_slot,
                              call.emit_cu, call.emit_pos, state_src=pool)


def to_device(arr):
    import torch
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(arr).cuda()


class GpuCall:
    """Device copies of a call's tensors plus its output and workspace buffers."""

    def __init__(self, call, pool, o_dtype="f32", scale=1.0, T_alloc=None, dst_pool=None):
        import torch
        from paper_2605_05219_amd import binding
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
        from paper_2605_05219_amd import binding
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
