"""Pins for the CPU oracle: checks it against things other than itself.

Each test targets a mistake that would otherwise go unseen: a dropped gate, the key
projection taken before instead of after the decay, a transposed state, an off-by-one in
the checkpoint position, a wrong head map, a wrong stride.
"""
import os

import numpy as np
import pytest

from oracle import gdn_oracle as orc
from paper_2605_05219_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_single(q, k, v, b, a, S0=None, emit=(), scale=1.0):
    """One layer, one head; arrays [T][d]; returns (o [T][d_v], states [n_emit][d_v][d_k])."""
    T = q.shape[0]
    f = lambda x: np.ascontiguousarray(x, dtype=np.float32)
    src = None if S0 is None else np.asarray(S0)[None, None, None]
    o, st = orc.resume_prefill(f(q)[None, :, None], f(k)[None, :, None], f(v)[None, :, None],
                               f(b)[None, :, None], f(a)[None, :, None],
                               [0, T], [0], [-1 if S0 is None else 0], [0, len(emit)], list(emit),
                               state_src=src, scale=scale)
    return o[0, :, 0], st[:, 0, 0]


def rand_inputs(rng, T, dk, dv):
    s = wl.token_streams(rng, 1, T, 1, 1, dk, dv, "f32")
    return tuple(x[0, :, 0].astype(np.float64) for x in (s.q, s.k, s.v)) + \
        (s.beta[0, :, 0].astype(np.float64), s.gate[0, :, 0].astype(np.float64))


# ------------------------------------------------------------------ worked example
def test_scalar_three_token_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "scalar_three_tokens.txt"))
            if l.strip() and not l.startswith("#")]
    a, b, v, q, s_exp, o_exp = (np.array([float(r[i]) for r in rows]) for i in range(1, 7))
    one = np.ones((3, 1))
    o, st = run_single(q[:, None], one, v[:, None], b, a, S0=np.array([[2.0]], dtype=np.float32),
                       emit=(1, 2, 3))
    assert np.array_equal(o[:, 0], o_exp)
    assert np.array_equal(st[:, 0, 0], s_exp)


# ------------------------------------------------------------------ brute force
def transition_product_reference(q, k, v, b, a, S0):
    """S_n = S_0 M_1..M_n + sum_t b_t v_t k_t^T M_{t+1}..M_n with M_t = a_t (I - b_t k_t k_t^T):
    the closed form of the recurrence, built from explicit d_k x d_k matrices."""
    T, dk = k.shape
    M = [a[t] * (np.eye(dk) - b[t] * np.outer(k[t], k[t])) for t in range(T)]
    outs = []
    for n in range(1, T + 1):
        tail = np.eye(dk)
        S = np.zeros_like(S0)
        for t in range(n - 1, -1, -1):
            S += b[t] * np.outer(v[t], k[t]) @ tail
            tail = M[t] @ tail
        S += S0 @ tail
        outs.append(S)
    return outs


@pytest.mark.parametrize("T,dk,dv", [(1, 1, 1), (5, 3, 2), (8, 4, 4), (7, 2, 5)])
def test_matches_transition_matrix_product(T, dk, dv):
    rng = np.random.default_rng(7 + T)
    q, k, v, b, a = rand_inputs(rng, T, dk, dv)
    S0 = rng.standard_normal((dv, dk)).astype(np.float32)
    o, st = run_single(q, k, v, b, a, S0=S0, emit=range(1, T + 1))
    ref = transition_product_reference(q, k, v, b, a, S0.astype(np.float64))
    for n in range(T):
        np.testing.assert_allclose(st[n], ref[n], rtol=0, atol=1e-13)
        np.testing.assert_allclose(o[n], ref[n] @ q[n], rtol=0, atol=1e-13)


def test_key_projection_uses_decayed_state():
    """One token: u = b (v - a S0 k), not b (v - S0 k)."""
    S0 = np.array([[2.0, 0.0], [0.0, 4.0]], dtype=np.float32)
    k = np.array([[1.0, 0.0]]); q = np.array([[1.0, 1.0]]); v = np.array([[1.0, 1.0]])
    o, st = run_single(q, k, v, np.array([0.5]), np.array([0.5]), S0=S0, emit=(1,))
    # a S0 = [[1,0],[0,2]]; a S0 k = [1,0]; u = .5([1,1]-[1,0]) = [0,.5]; S = [[1,0],[.5,2]]
    assert np.array_equal(st[0], np.array([[1.0, 0.0], [0.5, 2.0]]))
    assert np.array_equal(o[0], np.array([1.0, 2.5]))


# ------------------------------------------------------------------ special cases
def test_identity_token_leaves_state_bitwise():
    rng = np.random.default_rng(3)
    q, k, v, b, a = rand_inputs(rng, 6, 8, 8)
    S0 = rng.standard_normal((8, 8)).astype(np.float32)
    o, st = run_single(q, k, v, np.zeros(6), np.ones(6), S0=S0, emit=(1, 6))
    assert np.array_equal(st[0], S0.astype(np.float64))
    assert np.array_equal(st[1], S0.astype(np.float64))
    np.testing.assert_allclose(o, (S0.astype(np.float64) @ q.T).T, rtol=0, atol=1e-15)


def test_beta_zero_is_pure_decay():
    rng = np.random.default_rng(4)
    q, k, v, b, a = rand_inputs(rng, 9, 4, 3)
    S0 = rng.standard_normal((3, 4)).astype(np.float32)
    o, st = run_single(q, k, v, np.zeros(9), a, S0=S0, emit=(9,))
    gam = np.cumprod(a)
    np.testing.assert_allclose(st[0], gam[-1] * S0, rtol=1e-14)
    np.testing.assert_allclose(o, gam[:, None] * (q @ S0.T.astype(np.float64)), rtol=1e-13, atol=1e-15)


def test_orthonormal_keys_store_values_exactly():
    """a = 1, b = 1, orthonormal keys: the delta rule is an exact key -> value store."""
    rng = np.random.default_rng(5)
    d = 8
    Q, _ = np.linalg.qr(rng.standard_normal((d, d)))
    k = Q.astype(np.float32).astype(np.float64)      # rows nearly orthonormal after fp32 rounding
    v = rng.standard_normal((d, 5))
    o, st = run_single(k, k, v, np.ones(d), np.ones(d), emit=(d,))
    np.testing.assert_allclose(st[0] @ k.T, v.astype(np.float32).T, atol=2e-6)
    # and reading with q_t = k_t right after writing returns v_t
    np.testing.assert_allclose(o, v.astype(np.float32), atol=2e-6)


def test_repeated_key_overwrites_value():
    """a = 1, b = 1, the same unit key twice: the second value replaces the first."""
    k = np.array([[0.6, 0.8], [0.6, 0.8]])
    v = np.array([[1.0, 2.0, 3.0], [-4.0, 5.0, 0.5]])
    o, st = run_single(k, k, v, np.ones(2), np.ones(2), emit=(2,))
    kk = k[0].astype(np.float32).astype(np.float64)
    np.testing.assert_allclose(st[0] @ kk, v[1], atol=1e-6)


def test_scale_multiplies_outputs_only():
    rng = np.random.default_rng(6)
    q, k, v, b, a = rand_inputs(rng, 5, 4, 4)
    o1, s1 = run_single(q, k, v, b, a, emit=(5,))
    o2, s2 = run_single(q, k, v, b, a, emit=(5,), scale=0.25)
    assert np.array_equal(o2, 0.25 * o1) and np.array_equal(s1, s2)


# ------------------------------------------------------------------ exactness invariant (Remark 1)
@pytest.mark.parametrize("gate_mode", ["config", "slow", "one"])
def test_resume_equals_full_bitwise(gate_mode):
    rng = np.random.default_rng(11)
    T, d = 96, 16
    s = wl.token_streams(rng, 1, T, 1, 1, d, d, "f32", gate_mode)
    full_o, full_st = orc.resume_prefill(*s.fields(), [0, T], [0], [-1], [0, T],
                                         list(range(1, T + 1)))
    for p in (1, 17, 64, 95):
        ss = s.slice(p, T)
        o, st = orc.resume_prefill(*ss.fields(), [0, T - p], [p], [0], [0, 1], [T],
                                   state_src=full_st[p - 1][None])
        assert np.array_equal(o, full_o[:, p:])
        assert np.array_equal(st[0], full_st[T - 1])


def test_resume_from_wrong_state_is_detected_next_to_the_resume_point():
    """With the configs' gates a state is forgotten within tens of tokens, so a check far
    from the resume point proves nothing: the first tokens after it are what shows a bad
    checkpoint."""
    rng = np.random.default_rng(12)
    T, d, p = 200, 16, 64
    s = wl.token_streams(rng, 1, T, 1, 1, d, d, "f32")
    full_o, full_st = orc.resume_prefill(*s.fields(), [0, T], [0], [-1], [0, 1], [p])
    ss = s.slice(p, T)
    bad_o, _ = orc.resume_prefill(*ss.fields(), [0, T - p], [p], [-1], [0, 0], [])
    err = np.abs(bad_o - full_o[:, p:]).max(axis=(0, 2, 3))
    assert err[0] > 1e-3                  # visible right after the resume point
    assert err[-1] < 1e-12                # and gone far from it


def test_split_anywhere_gives_the_same_result():
    """oracle(x_1..n) = oracle(x_m+1..n) after oracle(x_1..m), for every m: pins 'the state at
    position c is the state after token c'."""
    rng = np.random.default_rng(13)
    T, d = 12, 4
    s = wl.token_streams(rng, 1, T, 1, 1, d, d, "f32")
    full_o, full_st = orc.resume_prefill(*s.fields(), [0, T], [0], [-1], [0, 1], [T])
    for m in range(1, T):
        _, st_m = orc.resume_prefill(*s.slice(0, m).fields(), [0, m], [0], [-1], [0, 1], [m])
        o2, st2 = orc.resume_prefill(*s.slice(m, T).fields(), [0, T - m], [m], [0], [0, 1], [T],
                                     state_src=st_m)
        assert np.array_equal(st2, full_st)
        assert np.array_equal(o2, full_o[:, m:])


# ------------------------------------------------------------------ layout, heads, dtypes
def test_grouped_value_heads_and_packing_match_single_head_runs():
    rng = np.random.default_rng(21)
    L, H_qk, H_v, dk, dv = 2, 2, 4, 4, 3
    lens = [5, 0, 7]
    T = sum(lens)
    s = wl.token_streams(rng, L, T, H_qk, H_v, dk, dv, "f32")
    pool = rng.standard_normal((3, L, H_v, dv, dk)).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)])
    start = [10, 4, 0]
    src = [2, 1, -1]
    emit_cu = [0, 2, 2, 3]
    emit_pos = [12, 15, 7]
    o, st = orc.resume_prefill(*s.fields(), cu, start, src, emit_cu, emit_pos, state_src=pool)
    for r in range(3):
        for l in range(L):
            for h in range(H_v):
                hq = h // (H_v // H_qk)
                sl = slice(cu[r], cu[r + 1])
                if lens[r] == 0:
                    continue
                S0 = pool[src[r], l, h] if src[r] >= 0 else None
                rel = [p - start[r] for p in emit_pos[emit_cu[r]:emit_cu[r + 1]]]
                o1, st1 = run_single(s.q[l, sl, hq], s.k[l, sl, hq], s.v[l, sl, h],
                                     s.beta[l, sl, h], s.gate[l, sl, h], S0=S0, emit=rel)
                assert np.array_equal(o[l, sl, h], o1)
                for j in range(len(rel)):
                    assert np.array_equal(st[emit_cu[r] + j, l, h], st1[j])


def test_state_is_dv_by_dk_row_major():
    """One token from zero: S = b v k^T, so S[i][j] = b v_i k_j (d_v rows, d_k columns)."""
    k = np.array([[0.5, 0.25, 1.0]]); v = np.array([[2.0, -4.0]]); q = np.array([[1.0, 0.0, 0.0]])
    o, st = run_single(q, k, v, np.array([0.5]), np.array([0.5]), emit=(1,))
    assert st.shape == (1, 2, 3)
    assert np.array_equal(st[0], 0.5 * np.outer(v[0], k[0]))


def test_bf16_inputs_are_widened_exactly():
    rng = np.random.default_rng(22)
    s16 = wl.token_streams(rng, 1, 20, 2, 2, 8, 8, "bf16")
    s32 = wl.Streams(*(wl.bf16_bits_to_f32(x) for x in s16.fields()))
    a = orc.resume_prefill(*s16.fields(), [0, 20], [0], [-1], [0, 1], [20])
    b = orc.resume_prefill(*s32.fields(), [0, 20], [0], [-1], [0, 1], [20])
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-39], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties to 1 + 2^-6
    bits = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5


# ------------------------------------------------------------------ Sec. 3 integer side
def test_deepest_checkpoint_brute_force():
    rng = np.random.default_rng(31)
    for _ in range(50):
        N = int(rng.integers(1, 60))
        M = int(rng.integers(0, min(N, 8) + 1))
        pos = sorted(rng.choice(np.arange(1, N + 1), size=M, replace=False).tolist())
        for t in range(0, N + 1):
            cands = [0] + [c for c in pos if c <= t]
            l = max(cands)
            i = orc.deepest_ckpt(pos, t)
            assert (pos[i] if i >= 0 else 0) == l
    assert orc.deepest_ckpt([128, 256, 384], 127) == -1
    assert orc.deepest_ckpt([128, 256, 384], 128) == 0      # c <= t: a checkpoint at t is reusable
    assert orc.deepest_ckpt([128, 256, 384], 512) == 2
    assert orc.deepest_ckpt([], 5) == -1


@pytest.mark.parametrize("N,M", [(512, 3), (8192, 16), (16384, 12), (32768, 8), (37, 5), (10, 10)])
def test_balanced_positions_meet_theorem_1(N, M):
    """Theorem 1: under uniform overlap a balanced set has
    E[r] = (1/N)((K-rho) q(q-1)/2 + rho q(q+1)/2) with N+1 = qK + rho, K = M+1,
    and worst-case recomputation ceil((N+1)/(M+1)) - 1."""
    pos = wl.balanced_positions(N, M)
    assert all(1 <= c <= N for c in pos) and all(x < y for x, y in zip(pos, pos[1:]))
    K = M + 1
    qq, rho = divmod(N + 1, K)
    expect = ((K - rho) * qq * (qq - 1) // 2 + rho * qq * (qq + 1) // 2)
    pos_arr = np.array([0] + pos)
    t = np.arange(1, N + 1)
    l = pos_arr[np.searchsorted(pos_arr, t, side="right") - 1]
    # spot-check the vectorised lookup against the oracle's own scan
    for tt in (1, pos[0] - 1 if pos[0] > 1 else 1, pos[0], N):
        i = orc.deepest_ckpt(pos, int(tt))
        assert (pos[i] if i >= 0 else 0) == l[tt - 1]
    r = t - l
    assert int(r.sum()) == expect                      # N E[r], exact integer
    assert int(r.max()) == -(-(N + 1) // (M + 1)) - 1


def test_config0_positions_are_the_balanced_ones():
    assert wl.balanced_positions(512, 3) == [128, 256, 384]


def test_gather_scatter_definitions():
    pool = np.arange(5 * 4, dtype=np.float32).reshape(5, 4)
    g = orc.ckpt_gather(pool, [3, -1, 0])
    assert np.array_equal(g, np.array([pool[3], np.zeros(4), pool[0]]))
    p2 = orc.ckpt_scatter(pool, [4, 1], g[:2])
    assert np.array_equal(p2[4], pool[3]) and np.array_equal(p2[1], np.zeros(4))
    assert np.array_equal(p2[[0, 2, 3]], pool[[0, 2, 3]])
