"""The attention layers' side of a cache hit (include/attn_resume.h) against the attention oracle.

CPU part: exports, argument validation.  GPU part (marked gpu): element by element through the
C ABI on bf16 inputs.  Tolerance on o: max |x - ref| <= 2e-3 max |ref| for the fp32 output, the bar
of the recurrence on bf16 inputs (here the weights enter the second contraction rounded to fp16,
relative error 2^-12 each, against a normaliser summed from the same rounded weights; everything
else is fp32, so the bar is met with an order of magnitude to spare), plus half a bf16 ulp
(2^-9 |ref| elementwise) when the output is stored as bf16.  Cache rows are copies (keys) or exact
widenings checked against numpy's float16 conversion (values): bit-exact.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import attn_oracle as ao
from paper_2605_05219_amd import attention as AT, binding as B, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_symbol_the_attention_header_declares():
    header = open(os.path.join(ROOT, "include", "attn_resume.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(attn_\w+)\s*\(", header))
    assert declared == set(AT.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None


class FakePool:
    """Stands in for a cache tensor [n_slots][cap][H_kv][d]: the checks under test return before any pointer is used."""

    def __init__(self, ptr=0x10000, n_slots=4, cap=512, stride0=512 * 2 * 64, nbytes=1 << 20):
        self._ptr, self.shape, self._s0, self._n = ptr, (n_slots, cap), stride0, nbytes

    def data_ptr(self): return self._ptr
    def stride(self, i): return self._s0
    def numel(self): return self._n
    def element_size(self): return 1


def prefill_args(**over):
    d = FakePool()
    a = dict(shape=AT.make_attn_shape(4, 2, 64), q=d, k_new=d, v_new=d, out_gate=None, cu_seqlens=[0, 100, 130], start_pos=[0, 64],
             k_cache=FakePool(ptr=0x200000), v_cache=FakePool(ptr=0x300000), seq_slot=[1, 3], o=d, workspace=FakePool(ptr=0x100000, nbytes=1 << 28))
    a.update(over)
    return a


@pytest.mark.parametrize("over,code", [
    (dict(shape=AT.make_attn_shape(4, 2, 96)), -3),
    (dict(shape=AT.make_attn_shape(4, 3, 64)), -3),                       # H_q not a multiple of H_kv
    (dict(shape=AT.make_attn_shape(4, 2, 64, scale=0.0)), -3),
    (dict(shape=AT.make_attn_shape(4, 2, 64, scale=float("nan"))), -3),
    (dict(cu_seqlens=[1, 100, 130]), -4),
    (dict(cu_seqlens=[0, 100, 90]), -4),
    (dict(start_pos=[-1, 64]), -10),
    (dict(start_pos=[0, 483]), -10),                                      # 483 + 30 rows do not fit cap = 512
    (dict(seq_slot=[1, 4]), -5),
    (dict(seq_slot=[-1, 2]), -5),
    (dict(seq_slot=[2, 2]), -6),
    (dict(q=FakePool(ptr=0)), -1),
    (dict(k_cache=FakePool(ptr=0)), -1),
    (dict(o=FakePool(ptr=0)), -1),
    (dict(k_new=FakePool(ptr=0x10008)), -2),
    (dict(out_gate=FakePool(ptr=0x10002)), -2),
    (dict(k_cache=FakePool(ptr=0x200000, stride0=512 * 2 * 64 + 4)), -2),
    (dict(k_cache=FakePool(ptr=0x200000, stride0=256 * 2 * 64)), -3),     # slots would overlap
    (dict(workspace=None), -9),
    (dict(workspace=FakePool(ptr=0x100000, nbytes=16)), -9),
])
def test_suffix_prefill_argument_errors(monkeypatch, over, code):
    """Every check fires on the host, before anything is enqueued."""
    monkeypatch.setattr(AT, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    a = prefill_args(**over)
    with pytest.raises(B.GdnError) as ei:
        AT.attn_suffix_prefill(a["shape"], a["q"], a["k_new"], a["v_new"], a["out_gate"], a["cu_seqlens"], a["start_pos"],
                               a["k_cache"], a["v_cache"], a["seq_slot"], a["o"], a["workspace"])
    assert ei.value.code == code


def test_restore_argument_errors_and_empty_calls(monkeypatch):
    monkeypatch.setattr(AT, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    sh, h, kc, vc = AT.make_attn_shape(4, 2, 64), FakePool(), FakePool(ptr=0x200000), FakePool(ptr=0x300000)
    for args, code in [((sh, [513, 1], h, h, [0, 1], kc, vc, [0, 1]), -10),          # a prefix longer than a slot
                       ((sh, [5, -1], h, h, [0, 1], kc, vc, [0, 1]), -10),
                       ((sh, [5, 1], h, h, [0, 4], kc, vc, [0, 1]), -5),
                       ((sh, [5, 1], h, h, [0, 1], kc, vc, [0, 7]), -5),
                       ((sh, [5, 1], h, h, [0, 1], kc, vc, [1, 1]), -6),
                       ((sh, [5, 1], FakePool(ptr=0), h, [0, 1], kc, vc, [0, 1]), -1),
                       ((sh, [5, 1], h, h, [0, 1], kc, FakePool(ptr=0x300008), [0, 1]), -2),
                       ((sh, [5, 1], FakePool(stride0=100), FakePool(stride0=100), [0, 1], kc, vc, [0, 1]), -2),
                       ((AT.make_attn_shape(4, 2, 32), [5, 1], h, h, [0, 1], kc, vc, [0, 1]), -3)]:
        with pytest.raises(B.GdnError) as ei:
            AT.attn_kv_restore(*args)
        assert ei.value.code == code
    with pytest.raises(B.GdnError) as ei:                                            # spill: two requests into one host slot
        AT.attn_kv_spill(sh, [5, 1], h, h, [2, 2], kc, vc, [0, 1])
    assert ei.value.code == -6
    AT.attn_kv_restore(sh, [], None, None, [], None, None, [])                       # nothing to do, nothing touched
    AT.attn_kv_restore(sh, [0, 0], h, h, [0, 0], kc, vc, [0, 1])                     # empty prefixes copy nothing
    AT.attn_suffix_prefill(sh, None, None, None, None, [0], [], None, None, [], None, None)
    AT.attn_suffix_prefill(sh, None, None, None, None, [0, 0, 0], [3, 3], kc, vc, [2, 2], None, None)   # empty requests only
    assert AT.attn_workspace_bytes(sh, 3, 1000) >= 4 * (3 * 3 + 1 + 9 * (1000 // 128 + 3)) + 768 * 128 * (64 + 2) * 4
    with pytest.raises(B.GdnError):
        AT.attn_workspace_bytes(sh, -1, 0)
    with pytest.raises(B.GdnError):
        AT.attn_workspace_bytes(AT.make_attn_shape(4, 2, 100), 1, 10)


def _check_plan(H_q, H_kv, d, lens, starts):
    """Invariants of the work list: every (token tile, key tile) a request needs is walked exactly once, parts of a
    split walk are consecutive ranges of whole tiles with consecutive slots, units come with the most tiles first."""
    sh = AT.make_attn_shape(H_q, H_kv, d)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    units, pack, kt = AT.attn_plan(sh, cu, starts)
    G = H_q // H_kv
    assert kt == (32 if d == 256 else 64) and pack in (1, G) and 128 % pack == 0
    tpw = 128 // pack
    spans = [int(u[3] - u[2]) for u in units]
    assert spans == sorted(spans, reverse=True) and all(x > 0 for x in spans)
    by_piece = {}
    for req, tile, t0, t1, part in units:
        by_piece.setdefault((int(req), int(tile)), []).append((int(t0), int(t1), int(part)))
    want_pieces = {(r, t) for r, n in enumerate(lens) for t in range(-(-n // tpw))}
    assert set(by_piece) == want_pieces
    slots = []
    for (r, t), parts in by_piece.items():
        parts.sort()
        kv = starts[r] + min((t + 1) * tpw, lens[r])
        assert parts[0][0] == 0 and parts[-1][1] == -(-kv // kt)
        assert all(a[1] == b[0] for a, b in zip(parts, parts[1:]))            # consecutive, no gap, no overlap
        if len(parts) == 1:
            assert parts[0][2] == -1
        else:
            ids = [p[2] for p in parts]
            assert ids == list(range(ids[0], ids[0] + len(ids)))              # consecutive workspace slots, in key order
            slots += ids
            # parts are balanced after the count is fixed from a target of at least 512 keys: none below two thirds of it
            assert min(p[1] - p[0] for p in parts) >= 1 and max(p[1] - p[0] for p in parts) * kt * 3 >= 512 * 2
    assert sorted(slots) == list(range(len(slots)))                           # slots are dense and distinct
    assert len(slots) * (H_q // pack) <= 768                                  # the partial results fit the workspace region
    return units, pack


def test_work_list_covers_every_tile_once_and_packs_and_splits_as_documented(monkeypatch):
    # long suffix, many workgroups: plain rows, whole walks
    u, pack = _check_plan(16, 2, 128, [8192], [0])
    assert pack == 1 and (u[:, 4] == -1).all() and len(u) == 64
    # short suffix behind a long prefix: packed rows (16 tokens x 8 heads), walks split into parts of 8 tiles
    u, pack = _check_plan(16, 2, 128, [64], [8000])
    assert pack == 8 and len(u) == 4 * 16 and (u[:, 3] - u[:, 2] <= 8).all()
    # 512 tokens: packing would not save rows; the walks are split
    u, pack = _check_plan(16, 2, 128, [512], [7680])
    assert pack == 1 and (u[:, 4] >= 0).all()
    # a group size that does not divide 128 is never packed; H_kv = 3 is fine for the planner
    _, pack = _check_plan(6, 2, 64, [5, 9], [100, 0])
    assert pack == 1
    # mixed batch, empty requests, d = 256 tiles of 32
    _check_plan(8, 1, 256, [0, 3, 200, 0, 129], [5, 4000, 64, 0, 1])
    _check_plan(4, 4, 64, [1] * 40, list(range(0, 4000, 100)))
    rng = np.random.default_rng(3)
    for _ in range(30):
        H_q, H_kv = [(4, 2), (16, 2), (8, 8), (32, 4), (12, 4)][rng.integers(5)]
        n = int(rng.integers(1, 9))
        _check_plan(H_q, H_kv, int(rng.choice([64, 128, 256])), [int(x) for x in rng.integers(0, 700, n)],
                    [int(x) for x in rng.integers(0, 9000, n)])
    # the switches
    try:
        AT.attn_tune_pack(False)
        assert _check_plan(16, 2, 128, [64], [8000])[1] == 1
        AT.attn_tune_split(False)
        u, _ = _check_plan(16, 2, 128, [64], [8000])
        assert (u[:, 4] == -1).all() and len(u) == 1
    finally:
        AT.attn_tune_pack(True)
        AT.attn_tune_split(True)
    # too small a capacity reports the count it needs
    sh = AT.make_attn_shape(16, 2, 128)
    with pytest.raises(B.GdnError) as ei:
        AT.attn_plan(sh, [0, 8192], [0], capacity=10)
    assert ei.value.code == -11


# ----------------------------------------------------------------------------- GPU parity
def f64(a):
    return wl.to_f32(a).astype(np.float64)


def oracle_o(c, scale, gate=False):
    out = np.zeros((c.T, c.H_q, c.d))
    for r in range(len(c.start_pos)):
        lo, hi = int(c.cu_seqlens[r]), int(c.cu_seqlens[r + 1])
        if hi > lo:
            out[lo:hi] = ao.attention_suffix(f64(c.q[lo:hi]), f64(c.k_full[r]), f64(c.v_full[r]), int(c.start_pos[r]), scale)
    return ao.output_gate(out, f64(c.gate)) if gate else out


def v_bits(v_bf16):
    """fp16 bit patterns of bf16 values, as the value cache holds them (numpy's round-to-nearest conversion)."""
    return wl.to_f32(v_bf16).astype(np.float16).view(np.uint16)


def pools_with_prefix(c, fill_k=0x7FC0, fill_v=0x7E00):
    """Cache pools [n_slots][cap][H_kv][d] as uint16 bits: NaN patterns everywhere, then each request's prefix rows."""
    k = np.full((c.n_slots, c.cap, c.H_kv, c.d), fill_k, np.uint16)
    v = np.full((c.n_slots, c.cap, c.H_kv, c.d), fill_v, np.uint16)
    for r, s in enumerate(c.seq_slot):
        p = int(c.start_pos[r])
        k[s, :p], v[s, :p] = c.k_full[r][:p], v_bits(c.v_full[r][:p])
    return k, v


def gpu_prefill(c, o_dtype="f32", gate=False, scale=None, pools=None):
    import torch
    from tests.harness import to_device
    sh = AT.make_attn_shape(c.H_q, c.H_kv, c.d, o_dtype, scale)
    kp, vp = pools if pools is not None else pools_with_prefix(c)
    k_cache, v_cache = to_device(kp), to_device(vp)
    o = torch.full((max(c.T, 1), c.H_q, c.d), float("nan"), dtype=torch.float32 if o_dtype == "f32" else torch.bfloat16, device="cuda")
    ws = torch.empty(AT.attn_workspace_bytes(sh, len(c.start_pos), c.T), dtype=torch.uint8, device="cuda")
    dev = lambda a: to_device(np.ascontiguousarray(a)) if a.size else None
    AT.attn_suffix_prefill(sh, dev(c.q), dev(c.suffix("k")), dev(c.suffix("v")), dev(c.gate) if gate else None, c.cu_seqlens,
                           c.start_pos, k_cache, v_cache, c.seq_slot, o, ws)
    torch.cuda.synchronize()
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    return o[:c.T].float().cpu().numpy().astype(np.float64), bits(k_cache), bits(v_cache)


def check_o(x, ref, o_dtype, what="o"):
    assert not np.isnan(x).any(), f"{what}: an element was never written"
    if ref.size == 0:
        return
    tol = 2e-3 * np.abs(ref).max() + (2.0 ** -9 * np.abs(ref) if o_dtype == "bf16" else 0.0)
    bad = np.abs(x - ref) > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} elements out, worst {np.abs(x - ref).max() / np.abs(ref).max():.3e} of max"


CASES = [
    # H_q, H_kv, d, lens, starts
    (4, 2, 64, [5], [0]),
    (4, 2, 64, [1], [0]),                                    # one token, one key
    (4, 2, 128, [300, 129, 1, 64], [0, 77, 500, 64]),        # several query tiles, ragged, a single-token suffix deep in a prefix
    (4, 1, 256, [200, 70], [130, 0]),
    (6, 3, 64, [150, 33], [10, 200]),                        # H_kv does not divide 8: the plain block order
    (16, 2, 128, [700], [1500]),                             # the grouping of the measured model family, 8 query heads per kv head
    (8, 8, 128, [128, 256, 127, 0, 65], [0, 64, 1, 9, 63]),  # exact tiles, an empty request, starts off the tile grid
    (2, 1, 64, [3, 2, 1, 4] * 16, [0, 1, 2, 70] * 16),       # many short requests
    (8, 4, 64, [70, 130], [33, 0]),                          # four key/value heads: two XCDs each in the block order
]


@pytest.mark.gpu
@pytest.mark.parametrize("case_i", range(len(CASES)))
@pytest.mark.parametrize("o_dtype,gate", [("f32", False), ("bf16", True)])
def test_suffix_attention_matches_the_oracle_and_appends_the_suffix(case_i, o_dtype, gate):
    H_q, H_kv, d, lens, starts = CASES[case_i]
    c = wl.attn_case(3000 + case_i, H_q, H_kv, d, lens, starts, spare_slots=2)
    got, k_after, v_after = gpu_prefill(c, o_dtype, gate)
    check_o(got, oracle_o(c, d ** -0.5, gate), o_dtype)
    # the caches: prefix rows as they were, suffix rows appended, every other row and slot untouched
    k_want, v_want = pools_with_prefix(c)
    for r, s in enumerate(c.seq_slot):
        k_want[s, :len(c.k_full[r])], v_want[s, :len(c.v_full[r])] = c.k_full[r], v_bits(c.v_full[r])
    assert np.array_equal(k_after, k_want) and np.array_equal(v_after, v_want)


@pytest.mark.gpu
def test_seeded_random_shapes_match_the_oracle():
    """Head groupings (also ones that cannot be packed or dealt to the XCDs), head sizes, request counts, lengths and
    starts drawn from a seeded generator: packed and plain rows, whole and split walks, ragged tiles in combinations the
    hand-picked cases do not list."""
    rng = np.random.default_rng(12345)
    heads = [(4, 2), (8, 1), (16, 2), (6, 3), (8, 8), (2, 2), (32, 4), (12, 4)]
    for it in range(24):
        H_q, H_kv = heads[rng.integers(len(heads))]
        d = int(rng.choice([64, 128, 256]))
        n_req = int(rng.integers(1, 7))
        lens = [int(x) for x in (rng.integers(0, 40, n_req) if it % 3 == 0 else rng.integers(0, 300, n_req) if it % 3 == 1
                                 else rng.choice([1, 16, 64, 127, 128, 129, 200], n_req))]
        starts = [int(x) for x in rng.choice([0, 1, 63, 64, 65, 500, 1023, 1024, 2500], n_req)]
        if sum(lens) == 0:
            lens[0] = 3
        o_dtype, gate = ("f32", False) if it % 2 == 0 else ("bf16", True)
        c = wl.attn_case(9000 + it, H_q, H_kv, d, lens, starts)
        got, k_after, v_after = gpu_prefill(c, o_dtype, gate)
        check_o(got, oracle_o(c, d ** -0.5, gate), o_dtype, f"case {it} {(H_q, H_kv, d, lens, starts)}")
        k_want, v_want = pools_with_prefix(c)
        for r, s in enumerate(c.seq_slot):
            k_want[s, :len(c.k_full[r])], v_want[s, :len(c.v_full[r])] = c.k_full[r], v_bits(c.v_full[r])
        assert np.array_equal(k_after, k_want) and np.array_equal(v_after, v_want), it


@pytest.mark.gpu
def test_peaked_and_flat_logits_stay_within_tolerance():
    """Widely spread logits (a few keys carry the weight; the running maximum moves often) and all-equal logits
    (every weight is exactly 1: the result is the running mean of the values to fp32 accuracy)."""
    c = wl.attn_case(3100, 4, 2, 128, [260, 90], [300, 0], q_spread=6.0)
    got, _, _ = gpu_prefill(c)
    check_o(got, oracle_o(c, 128 ** -0.5), "f32", "peaked")
    c = wl.attn_case(3101, 4, 2, 128, [200], [100])
    for r in range(1):
        c.k_full[r][:] = c.k_full[r][0]                    # identical keys: uniform weights over the visible positions
    got, _, _ = gpu_prefill(c, scale=0.37)
    ref = oracle_o(c, 0.37)
    check_o(got, ref, "f32", "flat")
    assert np.abs(got - ref).max() <= 2e-5 * np.abs(ref).max()     # no bf16 weight error at all in this case


@pytest.mark.gpu
def test_split_key_walks_agree_with_whole_walks(monkeypatch):
    """A call with few workgroups splits its long key walks and merges the parts: the same result up to the
    rounding of the fp16 weights (taken against another running maximum: 2^-12 relative each), also when parts
    lie wholly past some queries' limits (a short request behind a long prefix, off the tile grid)."""
    for seed, H_q, H_kv, d, lens, starts in [(3500, 4, 2, 128, [40, 300], [2000, 1111]), (3501, 2, 1, 64, [1, 129], [4095, 1500]),
                                             (3502, 2, 2, 256, [70], [1300]),
                                             (3503, 4, 2, 128, [100, 64, 0, 200], [0, 3000, 5, 900])]:   # whole and split walks in one call
        c = wl.attn_case(seed, H_q, H_kv, d, lens, starts)
        AT.attn_tune_split(False)
        try:
            whole, _, _ = gpu_prefill(c, gate=True)
        finally:
            AT.attn_tune_split(True)
        split, _, _ = gpu_prefill(c, gate=True)
        assert not np.array_equal(whole, split)                       # the split path did run
        assert np.abs(whole - split).max() <= 2.0 ** -11 * np.abs(whole).max()
        check_o(split, oracle_o(c, d ** -0.5, True), "f32")


@pytest.mark.gpu
def test_rows_packed_by_head_group_give_bitwise_the_unpacked_result(monkeypatch):
    """Short suffixes put the query heads of a key/value group into one workgroup's rows; a row's arithmetic does not
    depend on the lane that carries it, so the outputs equal the one-head-per-workgroup run bit for bit (walks under
    1024 keys, so neither run splits them), and a packed call with split walks still matches the oracle."""
    for seed, H_q, H_kv, d, lens, starts in [(3600, 8, 2, 128, [5, 40, 1, 33], [100, 300, 700, 0]), (3601, 16, 2, 64, [17, 64], [900, 13]),
                                             (3602, 4, 1, 256, [31, 2], [64, 500])]:
        c = wl.attn_case(seed, H_q, H_kv, d, lens, starts)
        AT.attn_tune_pack(False)
        try:
            plain, k1, v1 = gpu_prefill(c, gate=True)
        finally:
            AT.attn_tune_pack(True)
        packed, k2, v2 = gpu_prefill(c, gate=True)
        assert np.array_equal(plain, packed) and np.array_equal(k1, k2) and np.array_equal(v1, v2)
        check_o(packed, oracle_o(c, d ** -0.5, True), "f32")
    c = wl.attn_case(3603, 16, 2, 128, [64, 3], [5000, 2100])          # packed rows and split walks together
    got, _, _ = gpu_prefill(c, "bf16", True)
    check_o(got, oracle_o(c, 128 ** -0.5, True), "bf16")


@pytest.mark.gpu
def test_resuming_at_c_reproduces_the_full_prefill_bit_for_bit():
    """Exact reuse on the attention side: the rows after c of a prefill from 0 equal a call resumed at c over the
    restored prefix, bitwise (key tiles sit on an absolute grid, so every query sees the same arithmetic)."""
    H_q, H_kv, d, N = 4, 2, 128, 450
    full = wl.attn_case(3200, H_q, H_kv, d, [N], [0])
    o_full, k_full, v_full = gpu_prefill(full)
    for cpos in (1, 64, 131, 449):
        res = wl.attn_case(3200, H_q, H_kv, d, [N], [0])
        res.q, res.gate = full.q[cpos:], full.gate[cpos:]
        res.cu_seqlens, res.start_pos = np.asarray([0, N - cpos], np.int32), np.asarray([cpos], np.int32)
        o_res, k_res, v_res = gpu_prefill(res)
        assert np.array_equal(o_res, o_full[cpos:])
        assert np.array_equal(k_res, k_full) and np.array_equal(v_res, v_full)


@pytest.mark.gpu
def test_calls_interleaved_on_two_side_streams_equal_the_default_stream_result():
    """Two requests' calls (each with its own caches, output and workspace) enqueued alternately on two side streams,
    several times over, give bit for bit what the same calls give on the default stream: the index arrays of the calls
    travel through a shared ring of staging buffers and must not mix."""
    import torch
    from tests.harness import to_device
    cases = [wl.attn_case(3700, 8, 2, 128, [150, 3], [700, 2100]), wl.attn_case(3701, 8, 2, 128, [64], [1500])]
    want = [gpu_prefill(c, gate=True)[0] for c in cases]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    sets = []
    for c in cases:
        sh = AT.make_attn_shape(c.H_q, c.H_kv, c.d, "f32")
        kp, vp = pools_with_prefix(c)
        sets.append(dict(sh=sh, c=c, k=to_device(kp), v=to_device(vp), q=to_device(c.q), kn=to_device(c.suffix("k")),
                         vn=to_device(c.suffix("v")), g=to_device(c.gate),
                         o=torch.full((c.T, c.H_q, c.d), float("nan"), dtype=torch.float32, device="cuda"),
                         ws=torch.empty(AT.attn_workspace_bytes(sh, len(c.start_pos), c.T), dtype=torch.uint8, device="cuda")))
    torch.cuda.synchronize()
    for rep in range(6):
        for s_, st in zip(sets, streams):
            c = s_["c"]
            AT.attn_suffix_prefill(s_["sh"], s_["q"], s_["kn"], s_["vn"], s_["g"], c.cu_seqlens, c.start_pos, s_["k"], s_["v"],
                                   c.seq_slot, s_["o"], s_["ws"], stream=st)
    torch.cuda.synchronize()
    for s_, w in zip(sets, want):
        assert np.array_equal(s_["o"].cpu().numpy().astype(np.float64), w)


@pytest.mark.gpu
def test_restore_from_a_pinned_host_pool_is_bitwise_and_feeds_the_prefill():
    import torch
    from tests.harness import to_device
    H_q, H_kv, d = 4, 2, 128
    c = wl.attn_case(3300, H_q, H_kv, d, [70, 10, 129], [200, 0, 33], cap=400, spare_slots=1)
    # host pool: its own slot numbering, prefixes inside, other rows a pattern that must not travel
    n_host = 5
    hk = np.full((n_host, c.cap, H_kv, d), 0x7FC0, np.uint16)
    hv = np.full((n_host, c.cap, H_kv, d), 0x7E00, np.uint16)
    host_slot = np.asarray([3, 0, 4], np.int32)
    for r, hs in enumerate(host_slot):
        p = int(c.start_pos[r])
        hk[hs, :p], hv[hs, :p] = c.k_full[r][:p], v_bits(c.v_full[r][:p])
    pin = lambda a: torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).pin_memory()
    host_k, host_v = pin(hk), pin(hv)
    marker = np.full((c.n_slots, c.cap, H_kv, d), 0x3F80, np.uint16)
    k_cache, v_cache = to_device(marker), to_device(marker)
    sh = AT.make_attn_shape(H_q, H_kv, d)
    AT.attn_kv_restore(sh, c.start_pos, host_k, host_v, host_slot, k_cache, v_cache, c.seq_slot)
    torch.cuda.synchronize()
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    k_want, v_want = marker.copy(), marker.copy()
    for r, s in enumerate(c.seq_slot):
        p = int(c.start_pos[r])
        k_want[s, :p], v_want[s, :p] = c.k_full[r][:p], v_bits(c.v_full[r][:p])
    assert np.array_equal(bits(k_cache), k_want) and np.array_equal(bits(v_cache), v_want)
    got, k_after, v_after = gpu_prefill(c, pools=(bits(k_cache), bits(v_cache)))
    check_o(got, oracle_o(c, d ** -0.5), "f32")
    # and back: the finished requests' rows (prefix + suffix) spilled to fresh host slots, bit for bit, nothing else
    back_k, back_v = pin(np.full_like(hk, 0x1111)), pin(np.full_like(hv, 0x1111))
    n_rows = [len(kf) for kf in c.k_full]
    AT.attn_kv_spill(sh, n_rows, back_k, back_v, [1, 2, 0], to_device(k_after), to_device(v_after), c.seq_slot)
    torch.cuda.synchronize()
    hb = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    for r, hs in enumerate([1, 2, 0]):
        assert np.array_equal(hb(back_k)[hs, :n_rows[r]], c.k_full[r]) and np.array_equal(hb(back_v)[hs, :n_rows[r]], v_bits(c.v_full[r]))
        assert (hb(back_k)[hs, n_rows[r]:] == 0x1111).all() and (hb(back_v)[hs, n_rows[r]:] == 0x1111).all()
    assert (hb(back_k)[3:] == 0x1111).all() and (hb(back_v)[3:] == 0x1111).all()


@pytest.mark.gpu
def test_suffix_attention_at_a_serving_shape_on_sampled_rows():
    """One long request at the measured model family's head grouping, checked on sampled (token, head) rows."""
    H_q, H_kv, d, start, n = 16, 2, 128, 3000, 2100
    c = wl.attn_case(3400, H_q, H_kv, d, [n], [start])
    got, _, _ = gpu_prefill(c)
    rng = np.random.default_rng(5)
    kf, vf = f64(c.k_full[0]), f64(c.v_full[0])
    for i in list(rng.integers(0, n, size=24)) + [0, n - 1]:
        for h in rng.integers(0, H_q, size=2):
            g = h // (H_q // H_kv)
            t = start + int(i) + 1
            ref = ao.attention_suffix(f64(c.q[i:i + 1, h:h + 1]), kf[:t, g:g + 1], vf[:t, g:g + 1], t - 1, d ** -0.5)[0, 0]
            assert np.abs(got[i, h] - ref).max() <= 2e-3 * max(np.abs(ref).max(), 0.05), (i, h)
