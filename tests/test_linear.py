"""The layers' projections (include/gdn_linear.h) against their oracle (the definition in fp64).

CPU part: exports, argument validation (every check returns before a pointer is used).  GPU part (marked gpu):
element by element through the C ABI.

Tolerance, derived from the arithmetic: a product of two bf16 numbers is exact in fp32, so the only errors are those of
the fp32 accumulation of K terms, |err| <= K u sum_k |x_k w_k| with u = 2^-23 (one unit per addition covers a matrix
core that truncates rather than rounds), plus u |y| for the bias addition; a bf16 output adds its one rounding,
2^-8 |ref| (a whole ulp step, so that a value next to a rounding boundary may fall either way).  The bound is taken
per element with sum_k |x_k w_k| from the oracle on the absolute values.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import linear_oracle as lo
from paper_2605_05219_amd import binding as B, linear as LN

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_symbol_the_linear_header_declares():
    header = open(os.path.join(ROOT, "include", "gdn_linear.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(gdn_linear\w*)\s*\(", header))
    assert declared == set(LN.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None


def raw(**over):
    a = dict(x_ptr=0x100000, ldx=256, w_ptr=0x200000, ldw=256, bias_ptr=0x300000, y_ptr=0x400000, ldy=512,
             out_dtype=B.GDN_BF16, T=100, N=512, K=256)
    a.update(over)
    return LN.gdn_linear_raw(**a)


@pytest.mark.parametrize("over,code", [
    (dict(T=-1), -11), (dict(N=-1), -11), (dict(K=-64), -11),
    (dict(out_dtype=7), -3),
    (dict(K=200), -3), (dict(K=0), -3),                    # k steps are 64 wide; an empty sum is not a projection
    (dict(ldx=128), -3), (dict(ldw=192), -3), (dict(ldy=256), -3),
    (dict(x_ptr=0), -1), (dict(w_ptr=0), -1), (dict(y_ptr=0), -1),
    (dict(x_ptr=0x100008), -2), (dict(w_ptr=0x200004), -2), (dict(y_ptr=0x400004), -2),
    (dict(y_ptr=0x400008, out_dtype=B.GDN_F32), -2),
    (dict(bias_ptr=0x300002), -2),
    (dict(ldx=260), -2), (dict(ldw=257), -2), (dict(ldy=514), -2),
    (dict(ldx=1 << 22), -11),                              # a 256-row tile would pass 2 GiB of byte offsets
])
def test_argument_errors_are_reported_before_any_launch(over, code):
    assert raw(**over) == code


def test_empty_problems_are_legal_and_touch_nothing():
    assert raw(T=0, x_ptr=0, y_ptr=0) == 0
    assert raw(N=0, w_ptr=0, y_ptr=0, ldy=0) == 0


def split_raw(**over):
    a = dict(widths=[512, 256, 16, 16], ptrs=[0x400000, 0x500000, 0x600000, 0x700000], lds=[512, 256, 16, 16], out_dtype=B.GDN_BF16,
             T=100, K=256, x_ptr=0x100000, ldx=256, w_ptr=0x200000, ldw=256, bias_ptr=0)
    a.update(over)
    plan = LN.SplitPlan(a["widths"], a["ptrs"], a["lds"])
    return LN.gdn_linear_split_raw(a["x_ptr"], a["ldx"], a["w_ptr"], a["ldw"], a["bias_ptr"], plan, a["out_dtype"], a["T"], a["K"])


@pytest.mark.parametrize("over,code", [
    (dict(widths=[8] * 9, ptrs=[0x400000] * 9, lds=[8] * 9), -11),             # more than 8 segments
    (dict(widths=[512, 0, 16, 16]), -3),                                      # an empty segment
    (dict(widths=[500, 268, 16, 16]), -2),                                    # an inner boundary inside a 16-byte piece
    (dict(lds=[512, 128, 16, 16]), -3),                                       # a leading dimension below the segment's width
    (dict(lds=[512, 258, 16, 16]), -2),
    (dict(ptrs=[0x400000, 0, 0x600000, 0x700000]), -1),
    (dict(ptrs=[0x400000, 0x500004, 0x600000, 0x700000]), -2),
    (dict(K=100), -3), (dict(T=-1), -11), (dict(x_ptr=0), -1),
])
def test_split_argument_errors_are_reported_before_any_launch(over, code):
    assert split_raw(**over) == code


def test_split_with_no_tokens_is_legal():
    assert split_raw(T=0) == 0


def test_tile_knob_round_trip():
    prev = LN.gdn_linear_tune(2)
    assert LN.gdn_linear_tune(7) == 2          # out of range = per call
    assert LN.gdn_linear_tune(prev) == -1


def test_python_binding_rejects_mismatched_tensors():
    import torch
    x = torch.zeros((4, 64), dtype=torch.bfloat16)
    w = torch.zeros((8, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        LN.gdn_linear(x, torch.zeros((8, 128), dtype=torch.bfloat16), None, torch.zeros((4, 8), dtype=torch.bfloat16))
    with pytest.raises(ValueError):
        LN.gdn_linear(x, w, None, torch.zeros((4, 9), dtype=torch.bfloat16))
    with pytest.raises(ValueError):
        LN.gdn_linear(x.float(), w, None, torch.zeros((4, 8), dtype=torch.bfloat16))
    with pytest.raises(ValueError):
        LN.gdn_linear(x, w, torch.zeros(8, dtype=torch.bfloat16), torch.zeros((4, 8), dtype=torch.bfloat16))
    with pytest.raises(ValueError):
        LN.gdn_linear(x, w, None, torch.zeros((4, 8), dtype=torch.float16))


# ------------------------------------------------------------------------------------------ GPU parity

def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (input generation only)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def draw(seed, T, N, K, bias):
    """Activations ~ N(0,1), weights ~ N(0, 1/K) (outputs of unit scale, as after a normalisation layer), bias ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    x = bf16_bits(rng.standard_normal((T, K), dtype=np.float32))
    w = bf16_bits(rng.standard_normal((N, K), dtype=np.float32) / np.sqrt(K))
    b = rng.standard_normal(N, dtype=np.float32) if bias else None
    return x, w, b


def bound(x, w, b, ref, K, out):
    s_abs = lo.linear(np.abs(lo._f64(x)), np.abs(lo._f64(w)))
    tol = K * 2.0 ** -23 * s_abs + 2.0 ** -23 * np.abs(ref) + 1e-30
    if out == "bf16":
        tol = tol + 2.0 ** -8 * np.abs(ref)
    return tol


def run_gpu(x, w, b, out, ldy=None, col0=0):
    import torch
    from paper_2605_05219_amd.device_call import to_device
    T, N = x.shape[0], w.shape[0]
    xd, wd = to_device(x), to_device(w)
    bd = to_device(b) if b is not None else None
    dt = torch.bfloat16 if out == "bf16" else torch.float32
    full = torch.full((T, ldy if ldy is not None else N), float("nan"), dtype=dt, device="cuda")
    y = full[:, col0:col0 + N]
    LN.gdn_linear(xd, wd, bd, y, None)
    torch.cuda.synchronize()
    return full.float().cpu().numpy().astype(np.float64)


@pytest.mark.gpu
@pytest.mark.parametrize("T,N,K,bias,out", [
    (1, 36, 64, False, "f32"),                 # one token, a fraction of a tile
    (128, 128, 64, True, "bf16"),              # exactly one tile, one k step
    (300, 200, 128, True, "f32"),              # ragged in both directions, several tiles
    (300, 200, 128, False, "bf16"),
    (257, 130, 2048, True, "bf16"),            # the in-projection's depth; a tail of one token and two outputs
    (515, 8224, 2048, False, "bf16"),          # the in-projection of the timed layer: [q k v | z | a b] of d_model 2048
    (515, 2048, 2048, True, "f32"),            # the out-projection
    (64, 131, 192, True, "bf16"),              # an output count that is no multiple of 4 is only legal with ldy % 4 == 0
])
@pytest.mark.parametrize("shape", [0, 1, 2, 3, -1])
def test_linear_against_the_definition(T, N, K, bias, out, shape):
    x, w, b = draw(T * 7 + N * 3 + K, T, N, K, bias)
    ref = lo.linear(x, w, b)
    ldy = (N + 3) // 4 * 4
    prev = LN.gdn_linear_tune(shape)
    try:
        y = run_gpu(x, w, b, out, ldy=ldy)
    finally:
        LN.gdn_linear_tune(prev)
    assert np.isnan(y[:, N:]).all()            # nothing written past the last output
    err = np.abs(y[:, :N] - ref)
    tol = bound(x, w, b, ref, K, out)
    assert (err <= tol).all(), f"worst excess {(err / tol).max():.3f} at {np.unravel_index((err / tol).argmax(), err.shape)}"


@pytest.mark.gpu
def test_output_may_be_a_column_slice_of_a_wider_buffer():
    T, N, K = 200, 256, 128
    x, w, b = draw(5, T, N, K, True)
    ref = lo.linear(x, w, b)
    y = run_gpu(x, w, b, "bf16", ldy=1024, col0=512)
    assert np.isnan(y[:, :512]).all() and np.isnan(y[:, 768:]).all()
    assert (np.abs(y[:, 512:768] - ref) <= bound(x, w, b, ref, K, "bf16")).all()


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [0, 2, 3])
@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_split_outputs_equal_the_whole_projection(shape, out):
    """The in-projection of a layer in one launch: [conv input | z | a | b] to four tensors of their own (the last boundary
    ragged), each segment against the oracle's columns, nothing written outside."""
    import torch
    from paper_2605_05219_amd.device_call import to_device
    T, K = 300, 128
    widths = [384, 128, 16, 12]
    N = sum(widths)
    x, w, b = draw(17, T, N, K, True)
    ref = lo.linear(x, w, b)
    dt = torch.bfloat16 if out == "bf16" else torch.float32
    fulls = [torch.full((T, wd + 8), float("nan"), dtype=dt, device="cuda") for wd in widths]
    ys = [f[:, 4:4 + wd] for f, wd in zip(fulls, widths)]
    prev = LN.gdn_linear_tune(shape)
    try:
        LN.gdn_linear_split(to_device(x), to_device(w), to_device(b), ys, None)
        torch.cuda.synchronize()
    finally:
        LN.gdn_linear_tune(prev)
    tol = bound(x, w, b, ref, K, out)
    c = 0
    for f, wd in zip(fulls, widths):
        got = f.float().cpu().numpy().astype(np.float64)
        assert np.isnan(got[:, :4]).all() and np.isnan(got[:, 4 + wd:]).all()
        assert (np.abs(got[:, 4:4 + wd] - ref[:, c:c + wd]) <= tol[:, c:c + wd]).all()
        c += wd


@pytest.mark.gpu
def test_strided_inputs():
    import torch
    from paper_2605_05219_amd.device_call import to_device
    T, N, K = 150, 96, 128
    x, w, b = draw(6, T, N, K, False)
    xw = np.zeros((T, 2 * K), np.uint16); xw[:, K:] = x; xw[:, :K] = 0x7FC0          # NaNs beside the operand
    ww = np.zeros((N, 3 * K), np.uint16); ww[:, K:2 * K] = w; ww[:, :K] = 0x7FC0; ww[:, 2 * K:] = 0x7FC0
    xd, wd = to_device(xw)[:, K:], to_device(ww)[:, K:2 * K]
    y = torch.empty((T, N), dtype=torch.float32, device="cuda")
    LN.gdn_linear(xd, wd, None, y, None)
    torch.cuda.synchronize()
    ref = lo.linear(x, w, None)
    assert (np.abs(y.cpu().numpy().astype(np.float64) - ref) <= bound(x, w, None, ref, K, "f32")).all()


@pytest.mark.gpu
def test_full_size_projection_on_sampled_tokens():
    """The in-projection at the serving step's token count (the launch configuration the layer-group timing uses),
    checked on sampled tokens the oracle computes one by one."""
    import torch
    T, N, K = 131072 + 77, 8224, 2048
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    x = torch.randn((T, K), device="cuda", generator=g).bfloat16()
    w = (torch.randn((N, K), device="cuda", generator=g) / K ** 0.5).bfloat16()
    y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    LN.gdn_linear(x, w, None, y, None)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.random.default_rng(3).integers(0, T, 96), [0, 127, 128, T - 78, T - 77, T - 1]]))
    bits = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    xs, ws = bits(x[torch.from_numpy(rows).cuda()]), bits(w)
    ref = lo.linear(xs, ws, None)
    got = y[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
    assert (np.abs(got - ref) <= bound(xs, ws, None, ref, K, "bf16")).all()
