"""The layer's elementwise front and back ends (include/gdn_layer.h) against the layer oracle.

CPU part: exports, argument validation.  GPU part (marked gpu): element by element through the
C ABI.  Tolerances, per tensor: fp32 outputs max |x - ref| <= 1e-5 max |ref| (fp32 arithmetic with
hardware exp and reciprocal against fp64); bf16 outputs |x - ref| <= 2^-8 |ref| + 1e-6 elementwise
(half a bf16 ulp of rounding plus the fp32 error); convolution states are copies: bit-exact.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import layer_oracle as lo
from paper_2605_05219_amd import binding as B, layer as LY, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_symbol_the_layer_header_declares():
    header = open(os.path.join(ROOT, "include", "gdn_layer.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(gdn_layer_\w+)\s*\(", header))
    assert declared == set(LY.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None


class FakeDev:
    """Stands in for a device tensor: the checks under test return before any pointer is used."""

    def __init__(self, ptr=0x10000, n0=8, stride0=3 * 384, nbytes=1 << 20):
        self._ptr, self.shape, self._s0, self._n = ptr, (n0,), stride0, nbytes

    def data_ptr(self): return self._ptr
    def stride(self, i): return self._s0
    def numel(self): return self._n
    def element_size(self): return 1


def inputs_args(**over):
    d = FakeDev()
    a = dict(shape=LY.make_layer_shape(2, 2, 64, 64, 4, "bf16", "bf16"), x_qkv=d, conv_w=d, conv_b=d, a_pre=d, b_pre=d, A_log=d,
             dt_bias=d, cu_seqlens=[0, 100, 130], start_pos=[0, 64], conv_src=FakeDev(), src_slot=[-1, 2], emit_cu=[0, 2, 3],
             emit_pos=[50, 100, 94], conv_dst=FakeDev(ptr=0x90000), emit_slot=[0, 1, 3], q=d, k=d, v=d, beta=d, gate=d,
             workspace=FakeDev(ptr=0x100000))
    a.update(over)
    return a


@pytest.mark.parametrize("over,code", [
    (dict(shape=LY.make_layer_shape(2, 2, 96, 64)), -3),
    (dict(shape=LY.make_layer_shape(2, 2, 64, 64, conv_k=5)), -3),
    (dict(shape=LY.make_layer_shape(2, 2, 64, 64, conv_k=1)), -3),
    (dict(shape=LY.make_layer_shape(1, 1, 128, 64)), -3),              # a q/k head would straddle rows of channel groups
    (dict(shape=LY.make_layer_shape(2, 2, 64, 64, qk_eps=-1.0)), -3),
    (dict(cu_seqlens=[1, 100, 130]), -4),
    (dict(cu_seqlens=[0, 100, 90]), -4),
    (dict(start_pos=[-1, 64]), -10),
    (dict(emit_pos=[50, 101, 94]), -8),                                 # beyond the request's end
    (dict(emit_pos=[50, 50, 94]), -8),                                  # not increasing
    (dict(emit_pos=[50, 100, 64]), -8),                                 # at the start position: nothing consumed yet
    (dict(src_slot=[-1, 8]), -5),
    (dict(src_slot=[-2, 2]), -5),
    (dict(emit_slot=[0, 1, 8]), -5),
    (dict(emit_slot=[0, 1, 1]), -6),
    (dict(conv_dst=FakeDev(), emit_slot=[0, 2, 3]), -7),                # same pool, an emit slot is a source slot
    (dict(x_qkv=FakeDev(ptr=0)), -1),
    (dict(conv_src=FakeDev(ptr=0)), -1),
    (dict(conv_dst=FakeDev(ptr=0)), -1),
    (dict(q=FakeDev(ptr=0x10008)), -2),
    (dict(conv_src=FakeDev(stride0=3 * 384 + 4)), -2),
    (dict(conv_src=FakeDev(stride0=2 * 384)), -3),                      # slot smaller than a state
    (dict(workspace=None), -9),
    (dict(workspace=FakeDev(ptr=0x100000, nbytes=16)), -9),
    (dict(shape=LY.make_layer_shape(2, 2, 64, 64, L=0)), -3),
    (dict(shape=LY.make_layer_shape(2, 2, 64, 64, L=2)), -3),             # a slot of 3 x 384 holds one layer's rows, not two
    (dict(shape=LY.make_layer_shape(2, 2, 64, 64, T_alloc=129)), -4),     # 130 tokens do not fit a plane of 129
    (dict(shape=LY.make_layer_shape(2, 2, 64, 64, T_alloc=-1)), -3),
])
def test_layer_inputs_argument_errors(monkeypatch, over, code):
    """Every check fires on the host, before anything is enqueued."""
    monkeypatch.setattr(LY, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    a = inputs_args(**over)
    with pytest.raises(B.GdnError) as ei:
        LY.gdn_layer_inputs(a["shape"], a["x_qkv"], a["conv_w"], a["conv_b"], a["a_pre"], a["b_pre"], a["A_log"], a["dt_bias"],
                            a["cu_seqlens"], a["start_pos"], a["conv_src"], a["src_slot"], a["emit_cu"], a["emit_pos"],
                            a["conv_dst"], a["emit_slot"], a["q"], a["k"], a["v"], a["beta"], a["gate"], a["workspace"])
    assert ei.value.code == code


def test_layer_output_argument_errors_and_empty_calls(monkeypatch):
    monkeypatch.setattr(LY, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    d, sh = FakeDev(), LY.make_layer_shape(2, 2, 64, 64)
    for args, code in [((sh, FakeDev(ptr=0), d, d, d, 4), -1), ((sh, d, d, FakeDev(ptr=0x10004), d, 4), -2), ((sh, d, d, d, d, -1), -11),
                       ((LY.make_layer_shape(2, 2, 64, 32), d, d, d, d, 4), -3)]:
        with pytest.raises(B.GdnError) as ei:
            LY.gdn_layer_output(*args)
        assert ei.value.code == code
    LY.gdn_layer_output(sh, None, None, None, None, 0)                  # nothing to do, nothing touched
    LY.gdn_layer_inputs(sh, None, None, None, None, None, None, None, [0], [], None, [], [0], [], None, [], None, None, None, None,
                        None, None)
    assert LY.gdn_layer_workspace_bytes(3, 5) >= 4 * (4 * 3 + 2 + 3 * 5)
    with pytest.raises(B.GdnError):
        LY.gdn_layer_workspace_bytes(-1, 0)


# ----------------------------------------------------------------------------- GPU parity
def f64(a):
    return wl.to_f32(a).astype(np.float64)


def oracle_inputs(c, qk_eps):
    return lo.layer_inputs(f64(c.x_qkv), c.conv_w, c.conv_b, f64(c.a_pre), f64(c.b_pre), c.A_log, c.dt_bias, c.H_qk, c.H_v, c.d_k,
                           c.d_v, c.cu_seqlens, c.start_pos, c.src_slot, f64(c.conv_pool), c.emit_cu, c.emit_pos, qk_eps)


def gpu_inputs(c, out_dtype, qk_eps, conv_b=True):
    import torch
    from tests.harness import to_device
    sh = LY.make_layer_shape(c.H_qk, c.H_v, c.d_k, c.d_v, c.K, c.dtype, out_dtype, "f32", qk_eps)
    tdt = torch.float32 if out_dtype == "f32" else torch.bfloat16
    T = c.T
    new = lambda *s: torch.full(s, float("nan"), dtype=tdt, device="cuda")
    q, k, v = new(T, c.H_qk, c.d_k), new(T, c.H_qk, c.d_k), new(T, c.H_v, c.d_v)
    beta, gate = new(T, c.H_v), new(T, c.H_v)
    pool = to_device(c.conv_pool)
    before = pool.clone()
    ws = torch.empty(max(LY.gdn_layer_workspace_bytes(len(c.start_pos), int(c.emit_pos.size)), 256), dtype=torch.uint8, device="cuda")
    dev = lambda a: to_device(np.ascontiguousarray(a)) if a.size else None
    LY.gdn_layer_inputs(sh, dev(c.x_qkv), dev(c.conv_w), dev(c.conv_b) if conv_b else None, dev(c.a_pre), dev(c.b_pre), dev(c.A_log),
                        dev(c.dt_bias), c.cu_seqlens, c.start_pos, pool, c.src_slot, c.emit_cu, c.emit_pos, pool, c.emit_slot,
                        q, k, v, beta, gate, ws)
    torch.cuda.synchronize()
    host = lambda t: t.float().cpu().numpy().astype(np.float64)
    bits = lambda t: (t.view(torch.int16) if t.dtype == torch.bfloat16 else t).cpu().numpy()
    return [host(t) for t in (q, k, v, beta, gate)], bits(pool), bits(before)


def check_tensor(x, ref, out_dtype, what):
    assert not np.isnan(x).any(), f"{what}: an element was never written"
    if out_dtype == "f32":
        err = np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-30) if ref.size else 0.0
        assert err <= 1e-5, f"{what}: {err:.3e}"
    else:
        bad = np.abs(x - ref) > 2.0 ** -8 * np.abs(ref) + 1e-6
        assert not bad.any(), f"{what}: {int(bad.sum())} elements beyond half a bf16 ulp, worst {np.abs(x - ref).max():.3e}"


CASES = [
    # H_qk, H_v, d_k, d_v, K, lens, starts, emits
    (2, 2, 64, 64, 4, [256], [0], [[128, 256]]),
    (2, 2, 64, 64, 4, [1, 2, 3, 5, 0, 70], [9, 0, 4, 0, 11, 300], [[10], [1, 2], [5, 7], [3], [], [301, 302, 303, 333, 370]]),
    (2, 4, 128, 128, 4, [97, 33, 200], [64, 0, 1000], [[65, 66, 161], [33], [1100, 1200]]),
    (1, 2, 64, 128, 3, [50, 31], [5, 0], [[6, 55], [1, 2, 31]]),
    (2, 2, 128, 64, 2, [45, 64], [0, 3], [[1, 45], [4, 67]]),
    (16, 16, 128, 128, 4, [700, 1300], [512, 0], [[1024, 1212], [512, 1024, 1300]]),
]


def _many_short_requests(n_req=257, seed=7):
    """Many short requests, some empty, each storing its last state: the request lookup and run counting at scale."""
    rng = np.random.default_rng(seed)
    lens = [int(x) for x in rng.integers(0, 41, size=n_req)]
    starts = [int(x) for x in rng.integers(0, 3, size=n_req) * 64]
    emits = [[s + l] if l > 0 else [] for s, l in zip(starts, lens)]
    return (2, 2, 64, 64, 4, lens, starts, emits)


CASES.append(_many_short_requests())


@pytest.mark.gpu
@pytest.mark.parametrize("case_i", range(len(CASES)))
@pytest.mark.parametrize("dtype,out_dtype", [("bf16", "bf16"), ("f32", "f32"), ("bf16", "f32")])
def test_layer_inputs_match_the_oracle(case_i, dtype, out_dtype):
    H_qk, H_v, d_k, d_v, K, lens, starts, emits = CASES[case_i]
    c = wl.layer_case(2000 + case_i, H_qk, H_v, d_k, d_v, K, dtype, lens, starts, emits)
    ref = oracle_inputs(c, 1e-6)
    got, pool_after, pool_before = gpu_inputs(c, out_dtype, 1e-6)
    for name, x, r in zip(("q", "k", "v", "beta", "gate"), got, ref[:5]):
        check_tensor(x, r, out_dtype, name)
    # convolution states: copies, bit-exact, in the slots assigned and nowhere else
    want = pool_before.copy()
    stor = wl.to_storage(ref[5].astype(np.float32), dtype)
    stor = stor.view(np.int16) if dtype == "bf16" else stor
    for e, s in enumerate(c.emit_slot):
        want[s] = stor[e]
    assert np.array_equal(pool_after, want)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,out_dtype", [("bf16", "bf16"), ("f32", "f32")])
def test_stacked_layers_in_one_call_equal_one_call_per_layer_bitwise(dtype, out_dtype):
    """L = 3 layers with their own inputs and parameters in one launch ([L][T_alloc][...] planes with spare rows, slots of
    [L][K-1][C]) give bit for bit what three single-layer calls give (those are checked against the oracle above), for
    the front end, its emitted convolution states, and the back end."""
    import torch
    from tests.harness import to_device
    H_qk, H_v, d_k, d_v, K = 2, 4, 128, 128, 4
    lens, starts, emits = [97, 0, 33, 200], [64, 5, 0, 1000], [[65, 66, 161], [], [33], [1100, 1200]]
    cs = [wl.layer_case(2600 + l, H_qk, H_v, d_k, d_v, K, dtype, lens, starts, emits) for l in range(3)]
    for c in cs[1:]:
        c.src_slot, c.emit_slot = cs[0].src_slot, cs[0].emit_slot
    singles = [gpu_inputs(c, out_dtype, 1e-6) for c in cs]
    L, T, Ta, C = 3, cs[0].T, cs[0].T + 7, cs[0].C
    sh = LY.make_layer_shape(H_qk, H_v, d_k, d_v, K, dtype, out_dtype, "f32", 1e-6, L=L, T_alloc=Ta)
    tdt = torch.float32 if out_dtype == "f32" else torch.bfloat16
    def planes(arrs, fill=0):                                  # [L][T_alloc][...] from per-layer [T][...]
        out = np.full((L, Ta) + arrs[0].shape[1:], fill, arrs[0].dtype)
        for l, a in enumerate(arrs):
            out[l, :T] = a
        return to_device(out)
    new = lambda *s_: torch.full(s_, float("nan"), dtype=tdt, device="cuda")
    q, k, v = new(L, Ta, H_qk, d_k), new(L, Ta, H_qk, d_k), new(L, Ta, H_v, d_v)
    beta, gate = new(L, Ta, H_v), new(L, Ta, H_v)
    pool = to_device(np.ascontiguousarray(np.stack([c.conv_pool for c in cs], axis=1)))     # [slots][L][K-1][C]
    ws = torch.empty(LY.gdn_layer_workspace_bytes(len(starts), int(cs[0].emit_pos.size)), dtype=torch.uint8, device="cuda")
    stack = lambda name: to_device(np.ascontiguousarray(np.stack([getattr(c, name) for c in cs])))
    LY.gdn_layer_inputs(sh, planes([c.x_qkv for c in cs]), stack("conv_w"), stack("conv_b"), planes([c.a_pre for c in cs]),
                        planes([c.b_pre for c in cs]), stack("A_log"), stack("dt_bias"), cs[0].cu_seqlens, cs[0].start_pos, pool,
                        cs[0].src_slot, cs[0].emit_cu, cs[0].emit_pos, pool, cs[0].emit_slot, q, k, v, beta, gate, ws)
    torch.cuda.synchronize()
    host = lambda t: t.float().cpu().numpy().astype(np.float64)
    bits = lambda t: (t.view(torch.int16) if t.dtype == torch.bfloat16 else t).cpu().numpy()
    for l in range(L):
        for got, want in zip((q, k, v, beta, gate), singles[l][0]):
            assert np.array_equal(host(got[l, :T]), want)
        assert np.array_equal(bits(pool)[:, l], singles[l][1])
    assert torch.isnan(q[:, T:].float()).all()                                              # spare rows of the planes stay untouched
    # back end on the same planes
    o = planes([c.o for c in cs])
    z = planes([c.z for c in cs])
    y = new(L, Ta, H_v, d_v)
    LY.gdn_layer_output(sh, o, z, stack("norm_w"), y, T)
    sh1 = LY.make_layer_shape(H_qk, H_v, d_k, d_v, K, dtype, out_dtype, "f32", 1e-6)
    for l in range(L):
        y1 = new(T, H_v, d_v)
        LY.gdn_layer_output(sh1, to_device(cs[l].o), to_device(cs[l].z), to_device(cs[l].norm_w), y1, T)
        torch.cuda.synchronize()
        assert np.array_equal(host(y[l, :T]), host(y1))


@pytest.mark.gpu
def test_layer_inputs_resume_equals_full_replay_bitwise_on_the_gpu():
    """A request resumed from the convolution state the full run stored reproduces the full run's outputs bit for bit."""
    H, d, K, N, p = 2, 128, 4, 300, 131
    full = wl.layer_case(77, H, H, d, d, K, "bf16", [N], [0], [[p, N]], n_src_slots=1)
    got_f, pool_f, _ = gpu_inputs(full, "f32", 1e-6)
    res = wl.layer_case(77, H, H, d, d, K, "bf16", [N], [0], [[p, N]], n_src_slots=1)
    res.x_qkv, res.a_pre, res.b_pre = full.x_qkv[p:], full.a_pre[p:], full.b_pre[p:]
    res.cu_seqlens, res.start_pos = np.asarray([0, N - p], np.int32), np.asarray([p], np.int32)
    res.conv_pool = pool_f.view(np.uint16).copy()
    res.src_slot = np.asarray([full.emit_slot[0]], np.int32)
    res.emit_cu, res.emit_pos, res.emit_slot = np.asarray([0, 1], np.int32), np.asarray([N], np.int32), np.asarray([0], np.int32)
    got_r, pool_r, _ = gpu_inputs(res, "f32", 1e-6)
    for a, b in zip(got_r, got_f):
        assert np.array_equal(a, b[p:])
    assert np.array_equal(pool_r[0], pool_f[full.emit_slot[1]])
    # and a wrong state is seen in the first K-1 tokens only
    res.conv_pool = res.conv_pool.copy()
    res.conv_pool[res.src_slot[0]] = 0
    got_z, _, _ = gpu_inputs(res, "f32", 1e-6)
    assert not np.array_equal(got_z[2][:K - 1], got_f[2][p:p + K - 1]) and np.array_equal(got_z[2][K - 1:], got_f[2][p + K - 1:])


@pytest.mark.gpu
def test_layer_inputs_without_bias_and_feeding_the_recurrence():
    """No bias pointer = zero bias; the bf16 q, k, v, beta, gate are what gdn_resume_prefill reads (unit-norm q, k)."""
    c = wl.layer_case(5, 2, 2, 128, 128, 4, "bf16", [130], [0], [[130]])
    c.conv_b = np.zeros_like(c.conv_b)
    ref = oracle_inputs(c, 1e-6)
    got, _, _ = gpu_inputs(c, "bf16", 1e-6, conv_b=False)
    for name, x, r in zip(("q", "k", "v", "beta", "gate"), got, ref[:5]):
        check_tensor(x, r, "bf16", name)
    assert np.allclose((got[0] ** 2).sum(-1), 1.0, atol=2e-2) and np.allclose((got[1] ** 2).sum(-1), 1.0, atol=2e-2)


@pytest.mark.gpu
@pytest.mark.parametrize("H_v,d_v,T", [(2, 64, 1), (3, 128, 77), (16, 128, 1000)])
@pytest.mark.parametrize("o_dtype,dtype,out_dtype", [("f32", "bf16", "bf16"), ("f32", "f32", "f32"), ("bf16", "bf16", "f32"), ("bf16", "f32", "bf16")])
def test_layer_output_matches_the_oracle(H_v, d_v, T, o_dtype, dtype, out_dtype):
    import torch
    from tests.harness import to_device
    c = wl.layer_case(31, H_v, H_v, d_v, d_v, 4, dtype, [T], [0], [[T]])
    o_st = wl.to_storage(c.o, o_dtype)
    ref = lo.output_norm_gate(f64(o_st), f64(c.z), c.norm_w, 1e-5)
    sh = LY.make_layer_shape(H_v, H_v, d_v, d_v, 4, dtype, out_dtype, o_dtype, 1e-6, 1e-5)
    y = torch.full((T, H_v, d_v), float("nan"), dtype=torch.float32 if out_dtype == "f32" else torch.bfloat16, device="cuda")
    LY.gdn_layer_output(sh, to_device(o_st), to_device(c.z), to_device(c.norm_w), y, T)
    torch.cuda.synchronize()
    check_tensor(y.float().cpu().numpy().astype(np.float64), ref, out_dtype, "y")


@pytest.mark.gpu
def test_whole_layer_resumed_from_both_checkpointed_states_matches_the_composed_oracles():
    """Front end -> resumed recurrence -> back end on the GPU against the composition of the two oracles, for the full
    run and for a request resumed at p from the matrix state AND the convolution state the full run stored.

    The composed reference rounds its fp64 front-end outputs to bf16 as the path does; where the GPU's fp32 front end
    rounds an element the other way (a one-ulp difference in an input of the recurrence) the outputs move by far less
    than the recurrence's own tolerance, so the bar is that tolerance: 2e-3 max-normalised on o, + 2^-8 on the bf16 y.
    """
    import torch
    from oracle import gdn_oracle as orc
    from tests.harness import to_device
    H, d, K, N, p = 2, 128, 4, 300, 128
    c = wl.layer_case(91, H, H, d, d, K, "bf16", [N], [0], [[p, N]], n_src_slots=1)
    scale = d ** -0.5

    # ---- reference: layer oracle -> bf16 -> recurrence oracle -> output oracle
    rq, rk, rv, rb, rg, _ = oracle_inputs(c, 1e-6)
    st = lambda a: wl.to_storage(a.astype(np.float32), "bf16")[None]
    o_ref, S_ref = orc.resume_prefill(st(rq), st(rk), st(rv), st(rb), st(rg), [0, N], [0], [-1], [0, 2], [p, N], scale=scale)
    y_ref = lo.output_norm_gate(o_ref[0], f64(c.z), c.norm_w, 1e-5)

    def run(x_lo, start, conv_pool, conv_src, S_pool, S_src, emit_pos, conv_emit, S_emit):
        T = N - x_lo
        lsh = LY.make_layer_shape(H, H, d, d, K, "bf16", "bf16", "f32", 1e-6, 1e-5)
        new = lambda *s: torch.full(s, float("nan"), dtype=torch.bfloat16, device="cuda")
        q, k, v, beta, gate = new(1, T, H, d), new(1, T, H, d), new(1, T, H, d), new(1, T, H), new(1, T, H)
        ws = torch.empty(max(LY.gdn_layer_workspace_bytes(1, len(emit_pos)), 256), dtype=torch.uint8, device="cuda")
        ecu = [0, len(emit_pos)]
        LY.gdn_layer_inputs(lsh, to_device(c.x_qkv[x_lo:]), to_device(c.conv_w), to_device(c.conv_b), to_device(c.a_pre[x_lo:]),
                            to_device(c.b_pre[x_lo:]), to_device(c.A_log), to_device(c.dt_bias), [0, T], [start], conv_pool, [conv_src],
                            ecu, emit_pos, conv_pool, conv_emit, q, k, v, beta, gate, ws)
        sh = B.make_shape(1, H, H, d, d, "bf16", "f32", T, scale)
        o = torch.full((1, T, H, d), float("nan"), dtype=torch.float32, device="cuda")
        pws = torch.empty(max(B.gdn_workspace_bytes(sh, 1, T, len(emit_pos)), 256), dtype=torch.uint8, device="cuda")
        B.gdn_resume_prefill(sh, q, k, v, beta, gate, [0, T], [start], S_pool, [S_src], ecu, emit_pos, S_pool, S_emit, o, pws)
        y = new(T, H, d)
        LY.gdn_layer_output(lsh, o, to_device(c.z[x_lo:]), to_device(c.norm_w), y, T)
        torch.cuda.synchronize()
        return o[0].cpu().numpy().astype(np.float64), y.float().cpu().numpy().astype(np.float64)

    from tests.harness import max_norm_err
    conv_pool = torch.zeros((4, K - 1, c.C), dtype=torch.bfloat16, device="cuda")
    S_pool = torch.zeros((4, 1, H, d, d), dtype=torch.float32, device="cuda")
    o_full, y_full = run(0, 0, conv_pool, -1, S_pool, -1, [p, N], [0, 1], [0, 1])
    assert max_norm_err(o_full, o_ref[0]) <= 2e-3 and max_norm_err(y_full, y_ref) <= 2e-3 + 2.0 ** -8
    assert max_norm_err(S_pool[0].cpu().numpy(), S_ref[0]) <= 2e-3 and max_norm_err(S_pool[1].cpu().numpy(), S_ref[1]) <= 2e-3
    assert np.array_equal(conv_pool[0].view(torch.int16).cpu().numpy(), c.x_qkv[p - (K - 1):p].view(np.int16))
    # ---- resumed at p from slots 0 (matrix state and convolution state), new states into slots 2
    o_res, y_res = run(p, p, conv_pool, 0, S_pool, 0, [N], [2], [2])
    assert max_norm_err(o_res, o_ref[0, p:]) <= 2e-3 and max_norm_err(y_res, y_ref[p:]) <= 2e-3 + 2.0 ** -8
    assert max_norm_err(o_res[:16], o_ref[0, p:p + 16]) <= 2e-3          # where a wrong start state would show
    assert max_norm_err(S_pool[2].cpu().numpy(), S_ref[1]) <= 2e-3
    assert torch.equal(conv_pool[2], conv_pool[1])
    # a resume that restores S but not the convolution rows is NOT exact: the first tokens differ visibly
    o_bad, _ = run(p, p, conv_pool, -1, S_pool, 0, [N], [3], [3])
    assert max_norm_err(o_bad[:K - 1], o_ref[0, p:p + K - 1]) > 1e-2
