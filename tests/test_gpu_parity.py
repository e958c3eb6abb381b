"""GPU parity: the HIP library against the fp64 oracle, element by element, through the C ABI.

Tolerances (max |x - ref| / max |ref| per tensor; a tensor is all outputs of one (request, layer, value head),
or one value head of one emitted state):
  fp32 inputs  1e-5       bf16 inputs, fp32 o  2e-3       bf16 o  2e-3 + 2^-8 (its own rounding)
Slot indexing is exact: a state lands in the slot it was assigned and no other slot changes.
"""
import numpy as np
import pytest

from oracle import gdn_oracle as orc
from paper_2605_05219_amd import workloads as wl
from tests.harness import GpuCall, max_norm_err, run_call_gpu, run_call_oracle, worst_head_err, worst_state_err

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}


def fill_pool_from_oracle(sc):
    """Cache entry built by the oracle: pool slots hold the fp32-rounded exact states."""
    pool = np.zeros((sc.n_slots,) + sc.build.slot_shape, np.float32)
    o, st = run_call_oracle(sc.build, pool)
    for e, s in enumerate(sc.build.emit_slot):
        pool[s] = st[e].astype(np.float32)
    return pool, o, st


def check_call(call, pool, tol, o_dtype="f32", scale=1.0, first_tokens=16):
    o_ref, st_ref = orc.resume_prefill(*call.streams.fields(), call.cu_seqlens, call.start_pos, call.src_slot,
                                       call.emit_cu, call.emit_pos, state_src=pool, scale=scale)
    o, pool_after = run_call_gpu(call, pool, o_dtype=o_dtype, scale=scale)
    T = call.total_tokens
    assert not np.isnan(o[:, :T]).any(), "an output row was never written"
    o_tol = tol + (2.0 ** -8 if o_dtype == "bf16" else 0.0)
    # every (request, layer, value head) is a tensor of its own: small outputs get no looser bar
    err_o, where = worst_head_err(o, o_ref[:, :T], call.cu_seqlens)
    assert err_o <= o_tol, f"o error {err_o:.3e} > {o_tol} at (request, layer, head) {where}"
    # the tokens right after each resume point are where a wrong start state shows
    for r in range(call.n_req):
        lo = int(call.cu_seqlens[r]); hi = min(lo + first_tokens, int(call.cu_seqlens[r + 1]))
        if hi > lo:
            e, where = worst_head_err(o[:, lo:hi], o_ref[:, lo:hi], [0, hi - lo])
            assert e <= o_tol, (f"request {r}: error {e:.3e} in the first tokens after the resume point, "
                                f"(layer, head) {where[1:]}")
    touched = set()
    worst = 0.0
    for e, s in enumerate(call.emit_slot):
        err = worst_state_err(pool_after[s], st_ref[e])
        worst = max(worst, err)
        assert err <= tol, f"emitted state {e} (slot {s}) error {err:.3e} > {tol}"
        touched.add(int(s))
    for s in range(pool.shape[0]):
        if s not in touched:
            assert np.array_equal(pool_after[s], pool[s]), f"slot {s} changed but was not a destination"
    return err_o, worst


# ------------------------------------------------------------------ checkpoint pool copies
@pytest.mark.parametrize("n_slots,elems,n", [(8, 64, 3), (40, 2 * 2 * 64 * 64, 17), (600, 4096 + 4, 300),
                                             (6, 16 * 128 * 128, 6)])
def test_ckpt_gather_scatter_bit_exact(n_slots, elems, n):
    import torch
    from paper_2605_05219_amd import binding as B
    rng = np.random.default_rng(n_slots)
    pool_np = rng.standard_normal((n_slots, elems)).astype(np.float32)
    pool_np.view(np.uint32)[0, :4] = [0x7fc00001, 0xff800000, 0x00000001, 0x80000000]  # NaN payload, -inf, denormal, -0
    ids = rng.choice(n_slots, size=n, replace=False).astype(np.int32)
    ids_g = ids.copy(); ids_g[n // 2] = -1
    pool = torch.from_numpy(pool_np).cuda()
    dst = torch.full((n, elems), 7.0, device="cuda")
    B.ckpt_gather(pool, ids_g, dst)
    exp = orc.ckpt_gather(pool_np, ids_g)
    assert np.array_equal(dst.cpu().numpy().view(np.uint32), exp.view(np.uint32))
    src_np = rng.standard_normal((n, elems)).astype(np.float32)
    B.ckpt_scatter(pool, ids, torch.from_numpy(src_np).cuda())
    exp_pool = orc.ckpt_scatter(pool_np, ids, src_np)
    assert np.array_equal(pool.cpu().numpy().view(np.uint32), exp_pool.view(np.uint32))


def test_ckpt_copy_strided_destination_and_empty():
    import torch
    from paper_2605_05219_amd import binding as B
    pool = torch.arange(10 * 32, dtype=torch.float32, device="cuda").reshape(10, 32)
    big = torch.zeros(4, 48, device="cuda")
    B.ckpt_gather(pool, [9, 0, 3, 3], big, state_elems=32)      # dst stride 48 > 32 elements
    got = big.cpu().numpy()
    assert np.array_equal(got[:, :32], pool.cpu().numpy()[[9, 0, 3, 3]]) and not got[:, 32:].any()
    B.ckpt_gather(pool, [], big[:0])
    B.ckpt_scatter(pool, [], big[:0])


# ------------------------------------------------------------------ config 0: fp32, the worked configuration
def test_config0_full_then_resume_fp32():
    sc = wl.config0(orc.deepest_ckpt)
    empty = np.zeros((sc.n_slots,) + sc.build.slot_shape, np.float32)
    check_call(sc.build, empty, TOL["f32"])
    pool, _, _ = fill_pool_from_oracle(sc)
    assert list(sc.resume.start_pos) == [256] and list(sc.resume.emit_pos) == [384, 512]
    check_call(sc.resume, pool, TOL["f32"])


@pytest.mark.parametrize("gate_mode", ["slow", "one"])
def test_config0_slow_decay_fp32(gate_mode):
    """States that survive the whole prefix: a wrong start state cannot hide behind forgetting."""
    sc = wl.config0(orc.deepest_ckpt, gate_mode=gate_mode)
    pool, _, _ = fill_pool_from_oracle(sc)
    check_call(sc.resume, pool, TOL["f32"])


def test_wrong_start_state_would_be_caught():
    """The comparison itself: feeding the oracle a zero start state moves the first tokens far
    beyond the tolerance (CPU only; shows the parity check has teeth)."""
    sc = wl.config0(orc.deepest_ckpt)
    pool, _, _ = fill_pool_from_oracle(sc)
    good, _ = run_call_oracle(sc.resume, pool)
    bad, _ = run_call_oracle(sc.resume, np.zeros_like(pool))
    assert max_norm_err(bad[:, :16], good[:, :16]) > 100 * TOL["bf16"]


# ------------------------------------------------------------------ bf16 inputs
@pytest.mark.parametrize("d,H_qk,H_v,L", [(128, 2, 2, 1), (64, 2, 2, 1), (128, 2, 4, 2), (64, 1, 2, 2)])
@pytest.mark.parametrize("gate_mode", ["config", "slow"])
def test_ragged_requests_bf16(d, H_qk, H_v, L, gate_mode):
    """Several requests of ragged length, unaligned start and emit positions, empty request,
    grouped value heads, stacked layers: spans several chunks and a ragged tail."""
    rng = np.random.default_rng(100 + d + H_v + L)
    lens = [200, 0, 65, 1, 130, 64]
    starts = [0, 77, 513, 9, 128, 1000]
    n_slots = 24
    pool = (rng.standard_normal((n_slots, L, H_v, d, d)) * 0.5).astype(np.float32)
    src = [-1, 3, 5, 5, -1, 7]
    emits = [[64, 100, 200], [], [513 + 65], [10], [128 + 64, 128 + 128, 128 + 129], []]
    per = [wl.token_streams(rng, L, n, H_qk, H_v, d, d, "bf16", gate_mode) for n in lens]
    slots, nxt = [], 10
    for e in emits:
        slots.append(list(range(nxt, nxt + len(e)))); nxt += len(e)
    call = wl.pack_call(L, H_qk, H_v, d, d, "bf16", per, starts, src, emits, slots, n_slots)
    check_call(call, pool, TOL["bf16"])


def test_destination_may_be_own_source_slot():
    rng = np.random.default_rng(7)
    d = 64
    pool = (rng.standard_normal((4, 1, 2, d, d)) * 0.5).astype(np.float32)
    per = [wl.token_streams(rng, 1, 100, 2, 2, d, d, "bf16", "slow")]
    call = wl.pack_call(1, 2, 2, d, d, "bf16", per, [40], [2], [[140]], [[2]], 4)
    check_call(call, pool, TOL["bf16"])


@pytest.mark.parametrize("n_req,fused", [(2, -1), (3, -1), (4, -1), (6, -1), (12, 0), (12, -1), (16, 0), (16, -1), (32, 0), (32, -1)])
def test_batch_sizes_cover_every_launch_shape(n_req, fused):
    """16 heads x n_req requests: 32 chains run the latency variant with the next slab's preparation sharing the
    recurrence's launch, 48 and 64 chains the latency variant with separate launches (the recurrence takes most of the chip),
    96 chains two value-head slices per workgroup fed through an LDS ring; with the fused kernel forbidden 192 and 256 chains
    run the register-staged kernel with two slices per workgroup and 512 chains the one with four; left to itself the library
    gives these three sizes (short chains) to the fused kernel."""
    from paper_2605_05219_amd import binding as B
    sc = wl.config2(orc.deepest_ckpt, seed=2000 + n_req, n_req=n_req, N=1024, M=4, tail=70)
    pool, _, _ = fill_pool_from_oracle(sc)
    prev = B.gdn_tune_fused(fused)
    try:
        check_call(sc.resume, pool, TOL["bf16"])
    finally:
        B.gdn_tune_fused(prev)


@pytest.mark.parametrize("n_req,dtype", [(1, "bf16"), (4, "bf16"), (6, "bf16"), (32, "bf16"), (3, "f32")])
@pytest.mark.parametrize("rounds", [1, 3])
def test_short_slabs_carry_the_state_bitwise(n_req, dtype, rounds):
    """Slabs of 1 or 3 chunk rounds: every recurrence variant hands its state from slab to slab
    through the workspace; outputs and emitted states equal the automatic setting's bit for bit
    (and so meet the oracle tolerance, checked on the forced run)."""
    from paper_2605_05219_amd import binding as B
    d = 128 if dtype == "bf16" else 64
    H = 16 if dtype == "bf16" else 2
    rng = np.random.default_rng(300 + n_req)
    lens = [int(x) for x in rng.integers(1, 400, size=n_req)]
    lens[0] = 333
    starts = [int(x) for x in rng.integers(0, 50, size=n_req)]
    n_slots = 2 * n_req + 2
    pool = (rng.standard_normal((n_slots, 1, H, d, d)) * 0.5).astype(np.float32)
    src = [(-1 if r % 3 == 0 else r % 2) for r in range(n_req)]
    emits = [[starts[r] + lens[r]] if r % 2 == 0 else [] for r in range(n_req)]
    emits[0] = [starts[0] + 100, starts[0] + 333]
    per = [wl.token_streams(rng, 1, n, H, H, d, d, dtype, "slow") for n in lens]
    slots, nxt = [], 2
    for e in emits:
        slots.append(list(range(nxt, nxt + len(e)))); nxt += len(e)
    call = wl.pack_call(1, H, H, d, d, dtype, per, starts, src, emits, slots, n_slots)
    o_auto, pool_auto = run_call_gpu(call, pool)
    prev = B.gdn_tune_slab_rounds(rounds)
    try:
        o_forced, pool_forced = run_call_gpu(call, pool)
        check_call(call, pool, TOL[dtype])
    finally:
        B.gdn_tune_slab_rounds(prev)
    assert np.array_equal(o_auto, o_forced)
    assert np.array_equal(pool_auto, pool_forced)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("H_qk,H_v,L,o_dtype", [(2, 2, 1, "f32"), (2, 4, 2, "bf16")])
def test_fused_and_two_kernel_paths_both_meet_the_oracle(mode, H_qk, H_v, L, o_dtype):
    """The fused kernel (one workgroup per chain, operands stay in LDS) and the two-kernel path,
    each forced in turn, on ragged requests with unaligned starts and emits, grouped value
    heads, stacked layers, an empty request and both output types."""
    from paper_2605_05219_amd import binding as B
    rng = np.random.default_rng(500 + H_v + L)
    d = 128
    lens = [333, 0, 65, 1, 130, 64, 700, 47]
    starts = [0, 77, 513, 9, 128, 1000, 5, 64]
    n_slots = 30
    pool = (rng.standard_normal((n_slots, L, H_v, d, d)) * 0.5).astype(np.float32)
    src = [-1, 3, 5, 5, -1, 7, 2, 1]
    emits = [[64, 100, 333], [], [513 + 65], [10], [128 + 64, 128 + 128, 128 + 130], [], [5 + 700], [64 + 47]]
    per = [wl.token_streams(rng, L, n, H_qk, H_v, d, d, "bf16", "slow") for n in lens]
    slots, nxt = [], 10
    for e in emits:
        slots.append(list(range(nxt, nxt + len(e)))); nxt += len(e)
    call = wl.pack_call(L, H_qk, H_v, d, d, "bf16", per, starts, src, emits, slots, n_slots)
    prev = B.gdn_tune_fused(mode)
    try:
        check_call(call, pool, TOL["bf16"], o_dtype=o_dtype, scale=0.5)
    finally:
        B.gdn_tune_fused(prev)


def test_bf16_output_and_scale():
    sc = wl.config1(orc.deepest_ckpt, seed=5, n_draws=2, N=1024, M=4, H=4, d=128)
    pool, _, _ = fill_pool_from_oracle(sc)
    check_call(sc.resume, pool, TOL["bf16"], o_dtype="bf16", scale=128 ** -0.5)
    check_call(sc.resume, pool, TOL["bf16"], o_dtype="f32", scale=0.25)


def test_unaligned_balanced_positions():
    """Table 1's Balanced positions floor(i (N+1)/(M+1)) are not block aligned (e.g. 481, 963, ...)."""
    N, M = 2048, 4
    pos = wl.balanced_positions(N, M)
    assert any(p % 64 for p in pos)
    sc = wl.config1(orc.deepest_ckpt, seed=9, n_draws=3, N=N, M=M, H=4, d=128, positions=pos)
    empty = np.zeros((sc.n_slots,) + sc.build.slot_shape, np.float32)
    check_call(sc.build, empty, TOL["bf16"])
    pool, _, _ = fill_pool_from_oracle(sc)
    check_call(sc.resume, pool, TOL["bf16"])


# ------------------------------------------------------------------ exactness and determinism on the GPU
def test_gpu_resume_equals_gpu_full_bitwise_when_chunk_aligned():
    """Remark 1 on the device: with the resume point on a chunk boundary the resumed run
    repeats the same arithmetic on the same bits, so outputs and states are identical."""
    import torch
    sc = wl.config1(orc.deepest_ckpt, seed=11, n_draws=1, N=2048, M=4, H=4, d=128, gate_mode="slow")
    empty = np.zeros((sc.n_slots,) + sc.build.slot_shape, np.float32)
    o_full, pool = run_call_gpu(sc.build, empty)
    # a request identical to the prefix, resumed from checkpoint 2 (position 1024), same emits
    pos = sc.positions
    call = wl.resume_call(sc.prefix, pos, sc.slots, [pos[1]], [2048], [None], orc.deepest_ckpt, len(pos) + 1,
                          sc.n_slots + 8, "bf16", wl.emit_downstream(pos))
    pool2 = np.zeros((sc.n_slots + 8,) + sc.build.slot_shape, np.float32)
    pool2[:sc.n_slots] = pool
    o_res, pool2_after = run_call_gpu(call, pool2)
    assert np.array_equal(o_res, o_full[:, pos[1]:])
    for e, s in enumerate(call.emit_slot):
        assert np.array_equal(pool2_after[s], pool[sc.slots[2 + e]])


def test_run_to_run_bitwise_determinism():
    import torch
    sc = wl.config2(orc.deepest_ckpt, seed=13, n_req=6, N=1024, M=4, tail=33)
    pool, _, _ = fill_pool_from_oracle(sc)
    a = run_call_gpu(sc.resume, pool)
    b = run_call_gpu(sc.resume, pool)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_calls_on_a_side_stream_and_interleaved_streams_are_bitwise_the_default_stream_result():
    """The library enqueues on the caller's stream only: a call on a side stream, and two calls with their own
    workspaces interleaved on two streams, give the default-stream result bit for bit."""
    import torch
    from tests.harness import GpuCall
    sc = wl.config2(orc.deepest_ckpt, seed=17, n_req=5, N=1024, M=4, tail=40)
    pool, _, _ = fill_pool_from_oracle(sc)
    ref_o, ref_pool = run_call_gpu(sc.resume, pool)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    g1, g2 = GpuCall(sc.resume, pool), GpuCall(sc.resume, pool)
    torch.cuda.synchronize()
    for _ in range(3):
        with torch.cuda.stream(s1):
            g1.run(s1)
        with torch.cuda.stream(s2):
            g2.run(s2)
    torch.cuda.synchronize()
    T = sc.resume.total_tokens
    for g in (g1, g2):
        assert np.array_equal(g.o[:, :T].float().cpu().numpy(), ref_o)
        assert np.array_equal(g.pool.cpu().numpy(), ref_pool)


def test_two_host_threads_calling_concurrently_get_the_single_thread_result():
    """Two host threads, each with its own stream, tensors and workspace, call the library at the same time (ctypes
    drops the interpreter lock during a call): the shared plan staging buffer and the one-time set-up are guarded, and
    every call's result is the single-thread result bit for bit."""
    import threading
    import torch
    from tests.harness import GpuCall
    scs = [wl.config2(orc.deepest_ckpt, seed=21 + i, n_req=3 + 2 * i, N=1024, M=4, tail=40) for i in range(2)]
    pools = [fill_pool_from_oracle(sc)[0] for sc in scs]
    refs = [run_call_gpu(sc.resume, pool) for sc, pool in zip(scs, pools)]
    calls = [GpuCall(sc.resume, pool) for sc, pool in zip(scs, pools)]
    streams = [torch.cuda.Stream() for _ in scs]
    torch.cuda.synchronize()
    errors = []

    def worker(i):
        try:
            for _ in range(25):
                calls[i].run(streams[i])
            streams[i].synchronize()
        except Exception as exc:   # surfaced below: an exception in a thread would otherwise be lost
            errors.append(exc)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for i, sc in enumerate(scs):
        T = sc.resume.total_tokens
        assert np.array_equal(calls[i].o[:, :T].float().cpu().numpy(), refs[i][0])
        assert np.array_equal(calls[i].pool.cpu().numpy(), refs[i][1])


# ------------------------------------------------------------------ the configurations at full size
def test_config1_full_size_build_and_resume():
    """N = 8192, 16 heads, d = 128, M = 16: the entry build (8192 tokens) and resumes at seeded
    depths, every element against the oracle."""
    sc = wl.config1(orc.deepest_ckpt, n_draws=4)
    empty = np.zeros((sc.n_slots,) + sc.build.slot_shape, np.float32)
    check_call(sc.build, empty, TOL["bf16"])
    pool, _, _ = fill_pool_from_oracle(sc)
    # the bench runs one request per call: check each draw as its own call as well as batched
    check_call(sc.resume, pool, TOL["bf16"])
    one = wl.config1(orc.deepest_ckpt, n_draws=1)
    check_call(one.resume, pool, TOL["bf16"])


def test_config2_shape_reduced():
    sc = wl.config2(orc.deepest_ckpt, n_req=24, N=4096, M=12)
    pool, _, _ = fill_pool_from_oracle(sc)
    check_call(sc.resume, pool, TOL["bf16"])


def test_config3_shape_reduced_grouped_heads():
    sc = wl.config3(orc.deepest_ckpt, n_req=12, N=4096, M=8, H_qk=4, H_v=8)
    pool, _, _ = fill_pool_from_oracle(sc)
    check_call(sc.resume, pool, TOL["bf16"])


def test_config4_shape_reduced_layer_group():
    rng = np.random.default_rng(4)
    call = wl.config4_call(n_req=24, L=3, H=4, n_slots=160, lo=64, hi=1500, emit_step=512)
    pool = (rng.standard_normal((call.n_slots,) + call.slot_shape) * 0.5).astype(np.float32)
    check_call(call, pool, TOL["bf16"])


# ------------------------------------------------------------------ decode step
def decode_streams(rng, L, n_req, H_qk, H_v, d, dtype, gate_mode):
    return wl.token_streams(rng, L, n_req, H_qk, H_v, d, d, dtype, gate_mode)


@pytest.mark.parametrize("d,H_qk,H_v,L,dtype,n_req", [
    (128, 2, 2, 1, "bf16", 1), (128, 2, 2, 1, "bf16", 5), (128, 2, 2, 1, "bf16", 300),      # 300: two launches
    (64, 2, 4, 2, "bf16", 1), (64, 2, 4, 2, "bf16", 5), (64, 2, 4, 2, "bf16", 300),
    (64, 2, 2, 1, "f32", 1), (64, 2, 2, 1, "f32", 5), (64, 2, 2, 1, "f32", 300),
    (128, 4, 8, 1, "bf16", 1), (128, 4, 8, 1, "bf16", 5),
    (128, 16, 16, 1, "bf16", 140), (64, 16, 32, 1, "f32", 270), (64, 8, 16, 2, "bf16", 270)])   # > 128 MiB of states: streamed (non-temporal) rows
def test_decode_step_matches_the_token_loop(d, H_qk, H_v, L, dtype, n_req):
    """Two decode steps in a row (the second reads the states the first wrote in place) against
    the oracle's token loop run over both tokens; fp32 arithmetic on exactly widened inputs,
    so the fp32 tolerance holds for bf16 inputs too.  Slots not named are untouched."""
    import torch
    from paper_2605_05219_amd import binding as B
    from tests.harness import to_device
    rng = np.random.default_rng(900 + d + H_v + n_req)
    n_slots = n_req + 3
    pool = (rng.standard_normal((n_slots, L, H_v, d, d)) * 0.5).astype(np.float32)
    slots = rng.permutation(n_slots)[:n_req].astype(np.int32)
    steps = [decode_streams(rng, L, n_req, H_qk, H_v, d, dtype, "slow") for _ in range(2)]
    # oracle: request r = tokens (step 0, step 1) of row r, starting from its slot, state emitted after both
    per = []
    for r in range(n_req):
        a, b = steps[0].slice(r, r + 1), steps[1].slice(r, r + 1)
        per.append(wl.concat_streams([a, b]))
    call = wl.pack_call(L, H_qk, H_v, d, d, dtype, per, [0] * n_req, [int(s) for s in slots],
                        [[2]] * n_req, [[int(s)] for s in slots], n_slots)
    o_ref, st_ref = orc.resume_prefill(*call.streams.fields(), call.cu_seqlens, call.start_pos, call.src_slot,
                                       call.emit_cu, call.emit_pos, state_src=pool, scale=0.5)
    dpool = torch.from_numpy(pool.copy()).cuda()
    shape = B.make_shape(L, H_qk, H_v, d, d, dtype, "f32", n_req, 0.5)
    outs = []
    for st in steps:
        q, k, v, beta, gate = (to_device(np.ascontiguousarray(x)) for x in st.fields())
        o = torch.full((L, n_req, H_v, d), float("nan"), dtype=torch.float32, device="cuda")
        B.gdn_decode_step(shape, q, k, v, beta, gate, dpool, slots, o)
        torch.cuda.synchronize()
        outs.append(o.cpu().numpy())
    after = dpool.cpu().numpy()
    o_ref = o_ref[:, :2 * n_req].reshape(L, n_req, 2, H_v, d)
    for t in range(2):
        assert not np.isnan(outs[t]).any()
        assert max_norm_err(outs[t], o_ref[:, :, t]) <= TOL["f32"]
    named = set(int(s) for s in slots)
    for e, s in enumerate(call.emit_slot):
        assert max_norm_err(after[s], st_ref[e]) <= TOL["f32"]
    for s in range(n_slots):
        if s not in named:
            assert np.array_equal(after[s], pool[s])


# ------------------------------------------------------------------ full-size configs, sampled requests
def check_call_sampled(call, pool, tol, sample):
    """GPU runs the whole call; the oracle replays only the sampled requests (same tokens, start
    states and emit lists) and those requests' outputs and emitted states are compared."""
    o, pool_after = run_call_gpu(call, pool)
    assert not np.isnan(o[:, :call.total_tokens]).any(), "an output row was never written"
    for r in sample:
        lo, hi = int(call.cu_seqlens[r]), int(call.cu_seqlens[r + 1])
        e0, e1 = int(call.emit_cu[r]), int(call.emit_cu[r + 1])
        sub = wl.pack_call(call.L, call.H_qk, call.H_v, call.d_k, call.d_v, call.dtype, [call.streams.slice(lo, hi)],
                           [int(call.start_pos[r])], [int(call.src_slot[r])], [list(call.emit_pos[e0:e1])],
                           [list(call.emit_slot[e0:e1])], pool.shape[0])
        o_ref, st_ref = orc.resume_prefill(*sub.streams.fields(), sub.cu_seqlens, sub.start_pos, sub.src_slot,
                                           sub.emit_cu, sub.emit_pos, state_src=pool)
        if hi > lo:
            err, where = worst_head_err(o[:, lo:hi], o_ref[:, :hi - lo], [0, hi - lo])
            assert err <= tol, f"request {r} ({hi - lo} tokens): o error {err:.3e} > {tol} at (layer, head) {where[1:]}"
            n16 = min(16, hi - lo)
            err, where = worst_head_err(o[:, lo:lo + n16], o_ref[:, :n16], [0, n16])
            assert err <= tol, f"request {r}: o error {err:.3e} in the first tokens after the resume point"
        for e in range(e1 - e0):
            s = int(call.emit_slot[e0 + e])
            err = worst_state_err(pool_after[s], st_ref[e])
            assert err <= tol, f"request {r}: emitted state {e} (slot {s}) error {err:.3e} > {tol}"
    dst = set(int(s) for s in call.emit_slot)
    for s in range(pool.shape[0]):
        if s not in dst:
            assert np.array_equal(pool_after[s], pool[s]), f"slot {s} changed but was not a destination"


def sample_requests(call, k, rng):
    lens = np.diff(call.cu_seqlens)
    picks = {int(np.argmax(lens)), int(np.argmin(lens))}
    picks.update(int(x) for x in rng.choice(call.n_req, size=min(k, call.n_req), replace=False))
    return sorted(picks)


def test_config2_full_size_sampled_requests():
    """configs[2] as specified (64 requests, N = 16384, M = 12, 16 heads, d = 128): 1024 chains,
    several slabs in the throughput variant.  Start states are seeded random states (any state
    is a valid resume point); six requests, the longest and the shortest among them, are
    checked element by element."""
    rng = np.random.default_rng(2002)
    sc = wl.config2(orc.deepest_ckpt)
    pool = (rng.standard_normal((sc.n_slots,) + sc.build.slot_shape) * 0.3).astype(np.float32)
    check_call_sampled(sc.resume, pool, TOL["bf16"], sample_requests(sc.resume, 4, rng))


def test_config3_full_size_sampled_requests():
    """configs[3] as specified (32 requests, N = 32768, 16 query/key heads shared by 32 value heads, M = 8):
    1024 chains of heavily imbalanced length on the fused kernel.  The longest request, the three shortest and four
    seeded others are checked element by element."""
    rng = np.random.default_rng(2003)
    sc = wl.config3(orc.deepest_ckpt)
    assert sc.resume.n_req == 32
    pool = (rng.standard_normal((sc.n_slots,) + sc.build.slot_shape) * 0.3).astype(np.float32)
    lens = np.diff(sc.resume.cu_seqlens)
    short = [int(i) for i in np.argsort(lens)[:3]]
    check_call_sampled(sc.resume, pool, TOL["bf16"], sorted(set(short + sample_requests(sc.resume, 4, rng))))


def compare_step_request(step, r, layers, start):
    """Request r of a device-generated serving step, the given layers, every head: copied to the host, through the oracle
    from the start state `start`, compared element by element (outputs, the first tokens after the resume point on their
    own, every emitted state)."""
    sub = step.host_request(r, layers)
    one = np.ascontiguousarray(start[None])                                  # a one-slot pool for the oracle
    o_ref, st_ref = orc.resume_prefill(*sub.streams.fields(), sub.cu_seqlens, sub.start_pos, [0], sub.emit_cu,
                                       sub.emit_pos, state_src=one)
    lo, hi = int(step.cu_seqlens[r]), int(step.cu_seqlens[r + 1])
    o = step.o[layers, lo:hi].cpu().numpy()
    err, where = worst_head_err(o, o_ref, [0, hi - lo])
    assert err <= TOL["bf16"], f"request {r} ({hi - lo} tokens): o error {err:.3e} at (layer, head) {where[1:]}"
    n16 = min(16, hi - lo)
    err, where = worst_head_err(o[:, :n16], o_ref[:, :n16], [0, n16])
    assert err <= TOL["bf16"], f"request {r}: o error {err:.3e} in the first tokens after the resume point"
    for e, s in enumerate(sub.emit_slot):
        got = step.pool[int(s)][layers].cpu().numpy()
        err = worst_state_err(got, st_ref[e])
        assert err <= TOL["bf16"], f"request {r}: emitted state {e} (slot {int(s)}) error {err:.3e}"
    return sub.total_tokens


def test_config4_full_size_sampled_against_the_oracle():
    """configs[4] as specified and as `bench.py` times it: 256 requests x 8 layers x 16 heads = 32768 chains in one
    fused launch (each workgroup walks about 64 chains one after the other), a 4096-slot pool of 32 GiB, inputs
    generated on the device.  The seeded subsample goes to the host and through the oracle: every layer and head of
    16 requests (the longest and the shortest among them), and layer 0 of all 256 requests; each (request, layer,
    head) is compared element by element, emitted states too, slot ids with ==.  Slots that are no destination must
    not change: a checksum of every slot's bits, and 48 seeded slots compared bit for bit."""
    import torch
    from paper_2605_05219_amd.device_call import config4_device
    step = config4_device()
    assert (step.n_req, step.L, step.H, step.n_slots) == (256, 8, 16, 4096)
    rng = np.random.default_rng(4004)
    dst = set(int(s) for s in step.emit_slot)
    assert len(dst) == step.n_emit and not dst & set(int(s) for s in step.src_slot)
    bits = step.pool.view(torch.int32)
    sum_before = bits.sum(dim=(1, 2, 3, 4), dtype=torch.int64).cpu().numpy()
    watch = [int(s) for s in rng.permutation([s for s in range(step.n_slots) if s not in dst])[:48]]
    watch_before = step.pool[watch].cpu().numpy()
    picks = {int(np.argmax(step.lens)), int(np.argmin(step.lens))}
    picks.update(int(x) for x in rng.choice(step.n_req, size=14, replace=False))
    start_states = {r: step.pool[int(step.src_slot[r])].cpu().numpy() for r in range(step.n_req)
                    if r in picks}
    start_l0 = step.pool[torch.from_numpy(step.src_slot.astype(np.int64)).cuda(), 0].cpu().numpy()   # layer 0 of every source

    step.run()
    torch.cuda.synchronize()

    sum_after = bits.sum(dim=(1, 2, 3, 4), dtype=torch.int64).cpu().numpy()
    for s in range(step.n_slots):
        if s not in dst:
            assert sum_before[s] == sum_after[s], f"slot {s} changed but was not a destination"
    assert np.array_equal(step.pool[watch].cpu().numpy(), watch_before)
    assert not torch.isnan(step.o).any(), "an output row was never written"

    all_layers = list(range(step.L))
    for r in sorted(picks):
        compare_step_request(step, r, all_layers, start_states[r])
    for r in range(step.n_req):
        if r not in picks:
            compare_step_request(step, r, [0], start_l0[r][None])


def test_grouped_heads_serving_step_pairs_chosen_by_the_library():
    """A serving step of configs[4]'s recipe with 8 query/key heads under 16 value heads: 128 requests x 4 layers = 8192
    chains, enough for the library to give two value heads of a query/key head one workgroup.  That choice is checked
    against the oracle on sampled requests (every layer and head), and bit for bit, over the whole output and every pool
    slot, against the same call with one head per workgroup."""
    import torch
    from paper_2605_05219_amd import binding as B
    from paper_2605_05219_amd.device_call import config4_device
    step = config4_device(seed=1044, n_req=128, L=4, n_slots=1024, H_qk=8)
    rng = np.random.default_rng(4044)
    picks = {int(np.argmax(step.lens)), int(np.argmin(step.lens))}
    picks.update(int(x) for x in rng.choice(step.n_req, size=3, replace=False))
    start_states = {r: step.pool[int(step.src_slot[r])].cpu().numpy() for r in picks}
    pool_before = step.pool.clone()
    step.run()                                   # the library's own choice
    torch.cuda.synchronize()
    assert not torch.isnan(step.o).any(), "an output row was never written"
    for r in sorted(picks):
        compare_step_request(step, r, list(range(step.L)), start_states[r])
    o_auto, pool_auto = step.o.clone(), step.pool.clone()
    for pair in (0, 1):
        step.pool.copy_(pool_before)
        step.o.fill_(float("nan"))
        prev = B.gdn_tune_fused_pair(pair)
        try:
            step.run()
            torch.cuda.synchronize()
        finally:
            B.gdn_tune_fused_pair(prev)
        assert torch.equal(step.o.view(torch.int32), o_auto.view(torch.int32)), f"pair mode {pair}"
        assert torch.equal(step.pool.view(torch.int32), pool_auto.view(torch.int32)), f"pair mode {pair}"


# ------------------------------------------------------------------ host tier
def test_host_tier_fetch_and_spill_bit_exact():
    import torch
    from paper_2605_05219_amd import binding as B
    rng = np.random.default_rng(77)
    elems = 2 * 64 * 64
    host = torch.from_numpy(rng.standard_normal((9, elems)).astype(np.float32)).pin_memory()
    dev = torch.zeros((12, elems + 8), dtype=torch.float32, device="cuda")[:, :elems]     # padded stride
    before = dev.cpu().numpy().copy()
    h_ids, d_ids = [8, 0, 3, 3], [1, 11, 5, 6]
    B.ckpt_fetch_host(host, h_ids, dev, d_ids, elems)
    torch.cuda.synchronize()
    after = dev.cpu().numpy()
    for h, d in zip(h_ids, d_ids):
        assert np.array_equal(after[d], host[h].numpy())
    for d in set(range(12)) - set(d_ids):
        assert np.array_equal(after[d], before[d])
    back = torch.zeros((5, elems), dtype=torch.float32).pin_memory()
    B.ckpt_spill_host(back, [4, 0], dev, [11, 5], elems)
    torch.cuda.synchronize()
    assert np.array_equal(back[4].numpy(), host[0].numpy()) and np.array_equal(back[0].numpy(), host[3].numpy())
    assert not back[1:4].numpy().any()


@pytest.mark.parametrize("n_req,pinned", [(1, True), (6, True), (6, False)])
def test_prefill_from_host_pool_equals_prefill_from_device_pool(n_req, pinned):
    """Start states in a host pool: pinned memory is fetched by workgroups riding under the first
    preparation launch, pageable memory is copied on the stream first; outputs and emitted
    states bitwise those of the device-pool call, and within tolerance of the oracle.  Called
    twice (the staging area is reused)."""
    import torch
    from paper_2605_05219_amd import binding as B
    rng = np.random.default_rng(60 + n_req)
    d, H, L = 128, 4, 1
    lens = [int(x) for x in rng.integers(40, 700, size=n_req)]
    starts = [int(x) for x in rng.integers(0, 90, size=n_req)]
    n_src, n_dst = 5, 2 * n_req
    src_pool = (rng.standard_normal((n_src, L, H, d, d)) * 0.4).astype(np.float32)
    src = [(-1 if r == 2 else int(rng.integers(0, n_src))) for r in range(n_req)]
    emits = [[starts[r] + lens[r] // 2, starts[r] + lens[r]] for r in range(n_req)]
    slots = [[2 * r, 2 * r + 1] for r in range(n_req)]
    per = [wl.token_streams(rng, L, n, H, H, d, d, "bf16", "slow") for n in lens]
    call = wl.pack_call(L, H, H, d, d, "bf16", per, starts, src, emits, slots, max(n_src, n_dst))
    o_ref, st_ref = orc.resume_prefill(*call.streams.fields(), call.cu_seqlens, call.start_pos, call.src_slot,
                                       call.emit_cu, call.emit_pos, state_src=src_pool)
    # device-pool run (source and destination pools kept apart so that both runs see the same inputs)
    dst_dev = torch.zeros((n_dst, L, H, d, d), dtype=torch.float32, device="cuda")
    g = GpuCall(call, torch.from_numpy(src_pool).cuda(), dst_pool=dst_dev)
    g.run(); torch.cuda.synchronize()
    o_dev, st_dev = g.o[:, :call.total_tokens].cpu().numpy(), dst_dev.cpu().numpy()
    # host-pool run
    host_pool = torch.from_numpy(src_pool.copy())
    if pinned:
        host_pool = host_pool.pin_memory()
    dst_host = torch.zeros_like(dst_dev)
    ws = torch.empty(B.gdn_workspace_bytes_host(g.shape, call.n_req, call.total_tokens, int(call.emit_pos.size)),
                     dtype=torch.uint8, device="cuda")
    for _ in range(2):
        g.o.fill_(float("nan")); dst_host.zero_()
        B.gdn_resume_prefill_host(g.shape, g.q, g.k, g.v, g.beta, g.gate, call.cu_seqlens, call.start_pos, host_pool,
                                  call.src_slot, call.emit_cu, call.emit_pos, dst_host, call.emit_slot, g.o, ws)
        torch.cuda.synchronize()
        assert np.array_equal(g.o[:, :call.total_tokens].cpu().numpy(), o_dev)
        assert np.array_equal(dst_host.cpu().numpy(), st_dev)
    assert max_norm_err(o_dev, o_ref[:, :call.total_tokens]) <= TOL["bf16"]
    for e, s in enumerate(call.emit_slot):
        assert max_norm_err(st_dev[s], st_ref[e]) <= TOL["bf16"]


@pytest.mark.gpu
@pytest.mark.parametrize("many", [False, True])
def test_seeded_random_calls_match_the_oracle(many):
    """Shapes, request counts, lengths (also empty), start positions, source slots and emit positions drawn from a seeded
    generator, with random start states: combinations the hand-picked cases do not list; `many` draws 5 to 21 requests of
    the 16-head shapes, i.e. 80 to 336 chains, across the boundaries between the kernel variants."""
    rng = np.random.default_rng(4242 if many else 777)
    shapes = [(1, 2, 2, 64), (1, 2, 4, 128), (2, 1, 2, 64), (1, 4, 4, 128), (1, 16, 16, 128), (3, 2, 2, 128), (1, 8, 16, 128)]
    for it in range(16):
        L, H_qk, H_v, d = shapes[rng.integers(len(shapes))]
        dtype = "bf16" if (it % 4 or d != 64) else "f32"
        big = H_v * L >= 16
        n_req = int(rng.integers(5, 22)) if (many and big) else int(rng.integers(1, 5 if big else 40))
        lens = [int(x) for x in (rng.integers(0, 200, n_req) if (it % 2 or many) else rng.integers(0, 500 if big else 900, n_req))]
        if sum(lens) == 0:
            lens[0] = 5
        starts = [int(x) for x in rng.choice([0, 0, 64, 100, 512, 1000], n_req)]
        n_src, nxt = 3, 3
        emits, eslots = [], []
        for s0, ln in zip(starts, lens):
            e = sorted(set(int(x) for x in rng.integers(s0 + 1, s0 + ln + 1, int(rng.integers(0, 4))))) if ln > 0 else []
            emits.append(e)
            eslots.append(list(range(nxt, nxt + len(e))))
            nxt += len(e)
        per_req = [wl.token_streams(rng, L, ln, H_qk, H_v, d, d, dtype, "slow" if it % 3 == 0 else "config") for ln in lens]
        src = [-1 if s0 == 0 else int(rng.integers(0, n_src)) for s0 in starts]
        call = wl.pack_call(L, H_qk, H_v, d, d, dtype, per_req, starts, src, emits, eslots, nxt + 1)
        pool = rng.standard_normal((nxt + 1,) + call.slot_shape).astype(np.float32) * 0.1
        check_call(call, pool, TOL[dtype], o_dtype="bf16" if it % 5 == 0 else "f32")


@pytest.mark.gpu
@pytest.mark.parametrize("pair", [0, 1])
def test_seeded_random_calls_on_the_fused_kernel(pair):
    """The fused kernel forced onto small seeded calls it would not be chosen for: both head sizes, one value head (an
    output row is then exactly as long as the output descriptor's last row), grouped value heads (one head per workgroup,
    and two heads of a query/key head per workgroup where the group size is even), chunks of 1 to 64 tokens, requests of
    length 0, several layers, emits anywhere, both output types."""
    from paper_2605_05219_amd import binding as B
    rng = np.random.default_rng(9090)
    shapes = [(1, 1, 1, 128), (1, 1, 2, 128), (2, 1, 1, 64), (1, 2, 4, 128), (3, 2, 2, 64), (1, 4, 4, 128), (2, 2, 8, 64),
              (1, 1, 1, 64), (1, 16, 16, 64)]
    prev = B.gdn_tune_fused(1)
    prev_pair = B.gdn_tune_fused_pair(pair)
    try:
        for it in range(18):
            L, H_qk, H_v, d = shapes[it % len(shapes)]
            n_req = int(rng.integers(1, 7))
            lens = [int(x) for x in rng.choice([0, 1, 2, 15, 16, 17, 63, 64, 65, 100, 129, 200], n_req)]
            if sum(lens) == 0:
                lens[0] = 3
            starts = [int(x) for x in rng.choice([0, 0, 64, 100, 512], n_req)]
            nxt, emits, eslots = 3, [], []
            for s0, ln in zip(starts, lens):
                e = sorted(set(int(x) for x in rng.integers(s0 + 1, s0 + ln + 1, int(rng.integers(0, 4))))) if ln > 0 else []
                emits.append(e)
                eslots.append(list(range(nxt, nxt + len(e))))
                nxt += len(e)
            per_req = [wl.token_streams(rng, L, ln, H_qk, H_v, d, d, "bf16", "slow" if it % 3 == 0 else "config") for ln in lens]
            src = [-1 if s0 == 0 else int(rng.integers(0, 3)) for s0 in starts]
            call = wl.pack_call(L, H_qk, H_v, d, d, "bf16", per_req, starts, src, emits, eslots, nxt + 1)
            pool = rng.standard_normal((nxt + 1,) + call.slot_shape).astype(np.float32) * 0.1
            check_call(call, pool, TOL["bf16"], o_dtype="bf16" if it % 2 else "f32")
    finally:
        B.gdn_tune_fused(prev)
        B.gdn_tune_fused_pair(prev_pair)


@pytest.mark.gpu
@pytest.mark.parametrize("d,H_qk,H_v", [(128, 2, 8), (128, 3, 6), (64, 1, 4)])
def test_head_pairs_in_one_workgroup_equal_single_heads_bitwise(d, H_qk, H_v):
    """Two value heads of a query/key head in one workgroup share only the staged q and k rows: every head's arithmetic is
    that of the one-head kernel, so outputs and stored states agree bit for bit (and the one-head kernel is compared with
    the oracle)."""
    from paper_2605_05219_amd import binding as B
    rng = np.random.default_rng(4242 + d + H_v)
    L, lens, starts = 2, [200, 64, 1, 333, 0, 129], [128, 0, 64, 0, 0, 256]
    nxt, emits, eslots = 3, [], []
    for s0, ln in zip(starts, lens):
        e = sorted(set(int(x) for x in rng.integers(s0 + 1, s0 + ln + 1, 3))) if ln > 0 else []
        emits.append(e)
        eslots.append(list(range(nxt, nxt + len(e))))
        nxt += len(e)
    per_req = [wl.token_streams(rng, L, ln, H_qk, H_v, d, d, "bf16") for ln in lens]
    src = [-1 if s0 == 0 else int(rng.integers(0, 3)) for s0 in starts]
    call = wl.pack_call(L, H_qk, H_v, d, d, "bf16", per_req, starts, src, emits, eslots, nxt + 1)
    pool = rng.standard_normal((nxt + 1,) + call.slot_shape).astype(np.float32) * 0.1
    prev = B.gdn_tune_fused(1)
    prev_pair = B.gdn_tune_fused_pair(0)
    try:
        check_call(call, pool, TOL["bf16"])
        o1, p1 = run_call_gpu(call, pool)
        B.gdn_tune_fused_pair(1)
        o2, p2 = run_call_gpu(call, pool)
    finally:
        B.gdn_tune_fused(prev)
        B.gdn_tune_fused_pair(prev_pair)
    assert np.array_equal(o1.view(np.uint32), o2.view(np.uint32))
    assert np.array_equal(p1.view(np.uint32), p2.view(np.uint32))


@pytest.mark.gpu
@pytest.mark.parametrize("d", [128, 64])
def test_fused_chains_drawn_from_the_counter_match_the_oracle_for_any_workgroup_count(d):
    """640 short chains (20 requests, some empty, x 2 layers x 16 heads) on the fused kernel with one workgroup per compute
    unit: the first two rounds of chains are dealt by workgroup number, the rest are drawn from the counter in memory while
    the kernel runs.  Checked against the oracle, and bit for bit against the same call with as many workgroups per compute
    unit as fit (another grid, another assignment of chains to workgroups)."""
    from paper_2605_05219_amd import binding as B
    rng = np.random.default_rng(6400 + d)
    L, H, n_req = 2, 16, 20
    lens = [int(x) for x in rng.choice([0, 1, 30, 64, 65, 100, 129, 200, 260], n_req)]
    lens[3] = 0
    starts = [int(x) for x in rng.choice([0, 64, 128], n_req)]
    nxt, emits, eslots = 3, [], []
    for s0, ln in zip(starts, lens):
        e = sorted(set(int(x) for x in rng.integers(s0 + 1, s0 + ln + 1, 2))) if ln > 0 else []
        emits.append(e)
        eslots.append(list(range(nxt, nxt + len(e))))
        nxt += len(e)
    per_req = [wl.token_streams(rng, L, ln, H, H, d, d, "bf16") for ln in lens]
    src = [-1 if s0 == 0 else int(rng.integers(0, 3)) for s0 in starts]
    call = wl.pack_call(L, H, H, d, d, "bf16", per_req, starts, src, emits, eslots, nxt + 1)
    pool = rng.standard_normal((nxt + 1,) + call.slot_shape).astype(np.float32) * 0.1
    prev = B.gdn_tune_fused(1)
    prev_n = B.gdn_tune_fused_per_cu(1)
    try:
        check_call(call, pool, TOL["bf16"])
        o1, p1 = run_call_gpu(call, pool)
        B.gdn_tune_fused_per_cu(8)
        o2, p2 = run_call_gpu(call, pool)
    finally:
        B.gdn_tune_fused(prev)
        B.gdn_tune_fused_per_cu(prev_n)
    assert np.array_equal(o1.view(np.uint32), o2.view(np.uint32))
    assert np.array_equal(p1.view(np.uint32), p2.view(np.uint32))


@pytest.mark.gpu
@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("fused", [0, 1])
def test_extreme_gates(fused, d):
    """Gates that forget within one token (a = 1e-30, below what the clamp of log a lets through unchanged), gates of
    exactly 1, and ordinary ones mixed token by token, with beta at 0 and 1 among them: the decay factors between blocks
    may underflow but must never turn into infinities or NaNs, and a forgotten state must really be gone."""
    from paper_2605_05219_amd import binding as B
    rng = np.random.default_rng(31337)
    L, H, n = 1, 2, 200
    st = wl.token_streams(rng, L, n, H, H, d, d, "bf16")
    gate = wl.to_f32(st.gate).copy()
    beta = wl.to_f32(st.beta).copy()
    pick = rng.integers(0, 4, gate.shape)
    gate[pick == 0] = 1e-30
    gate[pick == 1] = 1.0
    gate[pick == 2] = 1e-3
    beta[rng.integers(0, 6, beta.shape) == 0] = 0.0
    beta[rng.integers(0, 6, beta.shape) == 0] = 1.0
    st = wl.Streams(st.q, st.k, st.v, wl.to_storage(beta, "bf16"), wl.to_storage(gate, "bf16"))
    call = wl.pack_call(L, H, H, d, d, "bf16", [st], [64], [1], [[100, 264]], [[2, 3]], 5)
    pool = (rng.standard_normal((5,) + call.slot_shape) * 0.5).astype(np.float32)
    prev = B.gdn_tune_fused(fused)
    try:
        check_call(call, pool, TOL["bf16"])
    finally:
        B.gdn_tune_fused(prev)


@pytest.mark.gpu
def test_probe_ceilings_reports_plausible_machine_rates():
    """The probe's figures lie between a fifth of the data-sheet peaks and the peaks themselves."""
    import torch
    from paper_2605_05219_amd import binding as B
    scratch = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    tf, gbs = B.gdn_probe_ceilings(scratch)
    assert 500.0 < tf < 2600.0, tf
    assert 1600.0 < gbs < 8100.0, gbs
