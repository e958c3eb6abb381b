"""CPU tests of the library's host side: exported symbols, l(t;C), the chunk planner and
every argument check of the entry points (all of them fire before anything is enqueued)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import gdn_oracle as orc
from paper_2605_05219_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gdn_resume.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(gdn_\w+|ckpt_\w+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None
    assert B.gdn_version() >= 100


def test_deepest_checkpoint_matches_brute_force():
    rng = np.random.default_rng(1)
    for _ in range(100):
        N = int(rng.integers(1, 80))
        M = int(rng.integers(0, min(N, 9) + 1))
        pos = sorted(rng.choice(np.arange(1, N + 1), size=M, replace=False).tolist())
        for t in range(0, N + 2):
            assert B.gdn_deepest_ckpt(pos, t) == orc.deepest_ckpt(pos, t)
    assert B.gdn_deepest_ckpt([128, 256, 384], 127) == -1
    assert B.gdn_deepest_ckpt([128, 256, 384], 128) == 0
    assert B.gdn_deepest_ckpt([], 7) == -1


def brute_plan(cu, start, ecu, epos):
    """Reference chunking written independently: walk positions one by one."""
    tok0, ln, em, rcu = [], [], [], [0]
    for r in range(len(start)):
        emits = {int(epos[e]): e for e in range(ecu[r], ecu[r + 1])}
        cur_start, cur_len = None, 0
        for i in range(cu[r + 1] - cu[r]):
            if cur_start is None:
                cur_start, cur_len = cu[r] + i, 0
            cur_len += 1
            pos = start[r] + i + 1
            if pos in emits or cur_len == B.GDN_CHUNK or i == cu[r + 1] - cu[r] - 1:
                tok0.append(cur_start); ln.append(cur_len); em.append(emits.get(pos, -1))
                cur_start = None
        rcu.append(len(tok0))
    return tok0, ln, em, rcu


def test_chunk_planner_matches_position_walk():
    rng = np.random.default_rng(2)
    for _ in range(60):
        n_req = int(rng.integers(1, 6))
        lens = rng.integers(0, 300, size=n_req)
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        start = rng.integers(0, 1000, size=n_req).astype(np.int32)
        epos, ecu = [], [0]
        for r in range(n_req):
            k = int(rng.integers(0, min(4, lens[r]) + 1))
            e = sorted(rng.choice(np.arange(1, lens[r] + 1), size=k, replace=False).tolist()) if k else []
            epos += [int(start[r] + x) for x in e]
            ecu.append(len(epos))
        got = B.gdn_plan_chunks(cu, start, ecu, epos)
        exp = brute_plan(cu, start, ecu, epos)
        for g, e in zip(got, exp):
            assert list(g) == list(e)


def test_chunk_planner_aligned_case():
    tok0, ln, em, rcu = B.gdn_plan_chunks([0, 256], [256], [0, 2], [384, 512])
    assert list(tok0) == [0, 64, 128, 192] and list(ln) == [64] * 4
    assert list(em) == [-1, 0, -1, 1] and list(rcu) == [0, 4]


@pytest.mark.parametrize("cu,start,ecu,epos,code", [
    ([1, 5], [0], [0, 0], [], -4),          # cu does not start at 0
    ([0, 5, 3], [0, 0], [0, 0, 0], [], -4), # decreasing
    ([0, 5], [-1], [0, 0], [], -10),        # negative start
    ([0, 5], [10], [0, 1], [10], -8),       # emit at the start position itself
    ([0, 5], [10], [0, 1], [16], -8),       # emit beyond the end
    ([0, 5], [10], [0, 2], [12, 12], -8),   # not strictly increasing
    ([0, 5], [10], [0, 2], [13, 12], -8),
    ([0, 5], [2**31 - 3], [0, 0], [], -10), # positions overflow int32
])
def test_chunk_planner_rejects(cu, start, ecu, epos, code):
    with pytest.raises(B.GdnError) as ei:
        B.gdn_plan_chunks(cu, start, ecu, epos, capacity=64)
    assert ei.value.code == code


def test_chunk_planner_capacity():
    with pytest.raises(B.GdnError) as ei:
        B.gdn_plan_chunks([0, 200], [0], [0, 0], [], capacity=3)
    assert ei.value.code == -9


def test_workspace_bytes_and_shape_checks():
    ok = B.make_shape(1, 16, 16, 128, 128, "bf16", "f32", 8192)
    n = B.gdn_workspace_bytes(ok, 1, 8192, 16)
    assert n > 0 and n % 256 == 0 or n > 0
    for bad in (B.make_shape(1, 3, 16, 128, 128, "bf16", "f32", 8),     # H_v % H_qk
                B.make_shape(1, 16, 16, 96, 96, "bf16", "f32", 8),      # head size
                B.make_shape(1, 16, 16, 64, 128, "bf16", "f32", 8),
                B.make_shape(0, 16, 16, 128, 128, "bf16", "f32", 8),
                B.make_shape(1, 2, 2, 128, 128, "f32", "f32", 8)):      # fp32 inputs: d = 64 only
        with pytest.raises(B.GdnError) as ei:
            B.gdn_workspace_bytes(bad, 1, 8, 0)
        assert ei.value.code == -3
    with pytest.raises(B.GdnError) as ei:
        B.gdn_workspace_bytes(ok, -1, 8, 0)
    assert ei.value.code == -11


class FakeDev:
    """Stands in for a device tensor: the checks under test return before any pointer is used."""

    def __init__(self, ptr=0x10000, n0=8, stride0=2 * 2 * 64 * 64, nbytes=1 << 30):
        self._ptr, self.shape, self._s0, self._n = ptr, (n0,), stride0, nbytes

    def data_ptr(self): return self._ptr
    def stride(self, i): return self._s0
    def dim(self): return 1
    def numel(self): return self._n
    def element_size(self): return 1
    def __getitem__(self, i): return self


def prefill_args(**over):
    shape = B.make_shape(1, 2, 2, 64, 64, "f32", "f32", 512)
    d = FakeDev()
    a = dict(shape=shape, q=d, k=d, v=d, beta=d, gate=d, cu_seqlens=[0, 256], start_pos=[256],
             state_src=d, src_slot=[1], emit_cu=[0, 2], emit_pos=[384, 512], state_dst=d,
             emit_slot=[3, 4], o=d, workspace=FakeDev(ptr=0x100000), stream=ctypes.c_void_p(0))
    a.update(over)
    return a


def call_prefill(monkeypatch, **over):
    monkeypatch.setattr(B, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    a = prefill_args(**over)
    B.gdn_resume_prefill(a["shape"], a["q"], a["k"], a["v"], a["beta"], a["gate"], a["cu_seqlens"],
                         a["start_pos"], a["state_src"], a["src_slot"], a["emit_cu"], a["emit_pos"],
                         a["state_dst"], a["emit_slot"], a["o"], a["workspace"], a["stream"])


@pytest.mark.parametrize("over,code", [
    (dict(src_slot=[8]), -5),                                   # source slot outside the pool
    (dict(src_slot=[-2]), -5),
    (dict(emit_slot=[3, 8]), -5),                               # destination outside the pool
    (dict(emit_slot=[3, -1]), -5),
    (dict(emit_slot=[3, 3]), -6),                               # duplicate destination
    (dict(cu_seqlens=[0, 100, 256], start_pos=[256, 0], src_slot=[1, 3], emit_cu=[0, 1, 2],
          emit_pos=[356, 156], emit_slot=[3, 4]), -7),          # request 0 writes request 1's source
    # the same hazard when the destination pool is a view of the source pool two slots further on (slots compared by address)
    (dict(cu_seqlens=[0, 100, 256], start_pos=[256, 0], src_slot=[1, 3], emit_cu=[0, 1, 2],
          emit_pos=[356, 156], emit_slot=[1, 4], state_dst=FakeDev(ptr=0x10000 + 2 * 4 * 2 * 2 * 64 * 64)), -7),
    # a destination that overlaps the writer's own source only partly (view shifted by half a slot)
    (dict(emit_slot=[0, 4], state_dst=FakeDev(ptr=0x10000 + 5 * 2 * 2 * 64 * 64)), -7),
    (dict(emit_pos=[384, 513]), -8),
    (dict(cu_seqlens=[0, 600], emit_pos=[384, 512]), -4),       # more tokens than T_alloc
    (dict(q=FakeDev(ptr=0)), -1),
    (dict(o=FakeDev(ptr=0x10004)), -2),
    (dict(state_src=FakeDev(ptr=0x10008)), -2),
    (dict(state_dst=FakeDev(stride0=2 * 64 * 64 - 4)), -3),      # slot stride smaller than a slot
    (dict(state_dst=FakeDev(stride0=2 * 64 * 64 + 2)), -2),      # slot stride not a multiple of 4 floats
    (dict(workspace=FakeDev(ptr=0x100010)), -9),                # not 256-byte aligned
    (dict(workspace=FakeDev(ptr=0x100000, nbytes=1024)), -9),   # too small
    (dict(state_src=FakeDev(ptr=0)), -1),
    (dict(state_src=None), -5),                                 # no source pool: slot 1 is out of range
])
def test_prefill_argument_errors(monkeypatch, over, code):
    with pytest.raises(B.GdnError) as ei:
        call_prefill(monkeypatch, **over)
    assert ei.value.code == code


def test_own_source_slot_may_be_a_destination(monkeypatch):
    """A request may overwrite the slot it started from; the hazard is only across requests.
    (Checked through a later error so that nothing reaches the device.)"""
    with pytest.raises(B.GdnError) as ei:
        call_prefill(monkeypatch, emit_slot=[1, 4], workspace=FakeDev(ptr=0x100000, nbytes=16))
    assert ei.value.code == -9


def test_empty_call_is_ok(monkeypatch):
    monkeypatch.setattr(B, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    shape = B.make_shape(1, 2, 2, 64, 64, "f32", "f32", 0)
    B.gdn_resume_prefill(shape, None, None, None, None, None, [0], [], None, [], [0], [], None, [], None, None,
                         ctypes.c_void_p(0))
    B.gdn_resume_prefill(shape, None, None, None, None, None, [0, 0], [5], None, [-1], [0, 0], [], None, [], None,
                         None, ctypes.c_void_p(0))


@pytest.mark.parametrize("fn", ["ckpt_gather", "ckpt_scatter"])
def test_copy_argument_errors(monkeypatch, fn):
    monkeypatch.setattr(B, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    f = getattr(B, fn)
    pool = FakeDev(n0=8, stride0=64)
    other = FakeDev(ptr=0x20000, n0=2, stride0=64)
    with pytest.raises(B.GdnError) as ei:
        f(pool, [0, 8], other, 64)
    assert ei.value.code == -5
    with pytest.raises(B.GdnError) as ei:
        f(pool, [0, 1], FakeDev(ptr=0x20004, stride0=64), 64)
    assert ei.value.code == -2
    with pytest.raises(B.GdnError) as ei:
        f(pool, [0, 1], other, 62)
    assert ei.value.code == -2
    with pytest.raises(B.GdnError) as ei:
        f(pool, [0, 1], other, 128)          # stride smaller than the state
    assert ei.value.code == -3
    if fn == "ckpt_scatter":
        with pytest.raises(B.GdnError) as ei:
            f(pool, [1, 1], other, 64)
        assert ei.value.code == -6
        with pytest.raises(B.GdnError) as ei:
            f(pool, [-1, 1], other, 64)
        assert ei.value.code == -5
    f(pool, [], other, 64)                    # nothing to copy: fine, nothing enqueued


def test_slab_rounds_knob_bounds_the_workspace():
    """A shorter slab needs a smaller workspace; the knob returns the previous setting."""
    shape = B.make_shape(1, 16, 16, 128, 128, "bf16", "f32", 8192)
    auto = B.gdn_workspace_bytes(shape, 1, 8192, 16)
    assert B.gdn_tune_slab_rounds(4) == 0
    try:
        small = B.gdn_workspace_bytes(shape, 1, 8192, 16)
        assert B.gdn_tune_slab_rounds(8) == 4
        mid = B.gdn_workspace_bytes(shape, 1, 8192, 16)
    finally:
        B.gdn_tune_slab_rounds(0)
    assert 0 < small < mid < auto
    assert B.gdn_workspace_bytes(shape, 1, 8192, 16) == auto


@pytest.mark.parametrize("over,code", [
    (dict(slot=[0, 0]), -6),                                   # two requests share a state
    (dict(slot=[0, 8]), -5),
    (dict(slot=[-1, 1]), -5),
    (dict(q=FakeDev(ptr=0)), -1),
    (dict(o=FakeDev(ptr=0x10004)), -2),
    (dict(pool=FakeDev(stride0=2 * 64 * 64 - 4)), -3),
    (dict(pool=FakeDev(stride0=2 * 64 * 64 + 2)), -2),
    (dict(slot=[0, 1, 2], T_alloc=2), -4),                      # more requests than token rows
])
def test_decode_argument_errors(monkeypatch, over, code):
    """Every check of gdn_decode_step fires on the host, before anything is enqueued."""
    monkeypatch.setattr(B, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    d = FakeDev()
    args = dict(q=d, k=d, v=d, beta=d, gate=d, pool=FakeDev(), slot=[0, 1], o=d, T_alloc=4)
    args.update(over)
    shape = B.make_shape(1, 2, 2, 64, 64, "f32", "f32", args.pop("T_alloc"))
    with pytest.raises(B.GdnError) as ei:
        B.gdn_decode_step(shape, args["q"], args["k"], args["v"], args["beta"], args["gate"], args["pool"], args["slot"],
                          args["o"], ctypes.c_void_p(0))
    assert ei.value.code == code


@pytest.mark.parametrize("fn", ["ckpt_fetch_host", "ckpt_spill_host"])
def test_host_tier_copy_argument_errors(monkeypatch, fn):
    monkeypatch.setattr(B, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    f = getattr(B, fn)
    host, dev = FakeDev(ptr=0x20000, n0=4, stride0=64), FakeDev(ptr=0x30000, n0=6, stride0=64)
    cases = [
        (dict(host_ids=[0, 4], dev_ids=[0, 1]), -5),
        (dict(host_ids=[0, 1], dev_ids=[0, 6]), -5),
        (dict(host_ids=[-1, 1], dev_ids=[0, 1]), -5),
        (dict(host_ids=[0, 1], dev_ids=[2, 2]) if fn == "ckpt_fetch_host" else dict(host_ids=[1, 1], dev_ids=[0, 2]), -6),
        (dict(host=FakeDev(ptr=0)), -1),
        (dict(dev=FakeDev(ptr=0x30004, n0=6, stride0=64)), -2),
        (dict(elems=66), -2),
        (dict(host=FakeDev(ptr=0x20000, n0=4, stride0=32)), -3),
    ]
    for over, code in cases:
        a = dict(host=host, dev=dev, host_ids=[0, 1], dev_ids=[0, 1], elems=64)
        a.update(over)
        with pytest.raises(B.GdnError) as ei:
            f(a["host"], a["host_ids"], a["dev"], a["dev_ids"], a["elems"], ctypes.c_void_p(0))
        assert ei.value.code == code, (over, ei.value.code)
    f(host, [], dev, [], 64, ctypes.c_void_p(0))                       # empty: nothing to do


def test_host_tier_workspace_is_the_device_one_plus_staging():
    shape = B.make_shape(1, 16, 16, 128, 128, "bf16", "f32", 8192)
    base = B.gdn_workspace_bytes(shape, 3, 8192, 16)
    assert B.gdn_workspace_bytes_host(shape, 3, 8192, 16) == (base + 255) // 256 * 256 + 3 * 16 * 128 * 128 * 4


@pytest.mark.parametrize("dev,code", [(FakeDev(ptr=0), -1), (FakeDev(ptr=0x10004), -2), (FakeDev(nbytes=1 << 19), -9)])
def test_probe_ceilings_argument_errors(monkeypatch, dev, code):
    """The machine-ceiling probe rejects a null, misaligned or too small scratch before touching the device."""
    monkeypatch.setattr(B, "_stream_ptr", lambda s=None: ctypes.c_void_p(0))
    with pytest.raises(B.GdnError) as ei:
        B.gdn_probe_ceilings(dev)
    assert ei.value.code == code


def test_headers_are_plain_c_and_a_c_program_can_call_the_library(tmp_path):
    """The boundary is a C ABI: the headers compile as strict C99 and a C program linked against the
    library calls host-only entry points through them."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "abi.c"
    src.write_text(
        '#include <stdio.h>\n#include "gdn_resume.h"\n#include "gdn_layer.h"\n#include "attn_resume.h"\n#include "ckpt_place.h"\n'
        "int main(void) {\n"
        "    const int32_t pos[3] = {128, 256, 384};\n"
        "    int32_t out[4];\n"
        "    gdn_shape s = {1, 2, 2, 64, 64, GDN_F32, GDN_F32, 1.0f, 512};\n"
        "    if (gdn_version() < 100) return 1;\n"
        "    if (gdn_deepest_ckpt(pos, 3, 300) != 1 || gdn_deepest_ckpt(pos, 3, 5) != -1) return 2;\n"
        "    if (gdn_workspace_bytes(&s, 1, 256, 2) <= 0) return 3;\n"
        "    if (gdn_layer_workspace_bytes(2, 3) <= 0) return 4;\n"
        "    attn_shape as = {16, 2, 128, GDN_BF16, 0.088f};\n"
        "    if (attn_workspace_bytes(&as, 2, 300) <= 0) return 6;\n"
        "    { const int32_t cu[2] = {0, 64}, st[1] = {8000}; int32_t u[5][64], nu, pk, kt;\n"
        "      if (attn_plan(&as, 1, cu, st, 64, u[0], u[1], u[2], u[3], u[4], &nu, &pk, &kt) != GDN_OK || nu != 64 || pk != 8 || kt != 64) return 7; }\n"
        "    if (ckpt_place_balanced(511, 3, out) != 3 || out[0] != 128 || out[2] != 384) return 5;\n"
        '    printf("ok\\n");\n    return 0;\n}\n')
    exe = tmp_path / "abi"
    pkg = os.path.dirname(B.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
                           str(src), "-o", str(exe), "-L", pkg, "-lgdn_resume", "-Wl,-rpath," + pkg])
    assert subprocess.run([str(exe)], capture_output=True, text=True).stdout.strip() == "ok"


def test_bench_refuses_more_than_one_gpu_with_a_message():
    """bench.py --gpus N with N above 1 exits at once with a message that says why (nothing touches a GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode == 2 and res.stdout == "" and "ONE GPU" in res.stderr
