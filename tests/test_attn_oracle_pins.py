"""Pins of the attention oracle against what the mathematics fixes: closed forms, invariants,
a scalar brute force written with explicit loops, and a library softmax.  CPU only."""
import math

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import attn_oracle as ao


def rand(rng, *shape):
    return rng.standard_normal(shape)


def test_a_single_visible_key_returns_its_value():
    rng = np.random.default_rng(0)
    q, k, v = rand(rng, 1, 4, 8), rand(rng, 1, 2, 8), rand(rng, 1, 2, 8)
    o = ao.attention_suffix(q, k, v, start=0, scale=0.3)
    for h in range(4):
        np.testing.assert_allclose(o[0, h], v[0, h // 2], rtol=0, atol=1e-15)


@pytest.mark.parametrize("start", [0, 1, 5])
def test_zero_queries_give_the_running_mean_of_the_values(start):
    # all logits equal: uniform weights over positions 1..t, so o_t is the prefix mean of v; an
    # off-by-one in the causal limit or a dropped start offset changes the count
    rng = np.random.default_rng(1)
    n, total = 6, start + 6
    q = np.zeros((n, 2, 4))
    k, v = rand(rng, total, 1, 4), rand(rng, total, 1, 4)
    o = ao.attention_suffix(q, k, v, start=start, scale=1.0)
    for i in range(n):
        t = start + i + 1
        want = v[:t, 0].mean(axis=0)
        np.testing.assert_allclose(o[i, 0], want, rtol=1e-13)
        np.testing.assert_allclose(o[i, 1], want, rtol=1e-13)


def test_two_keys_closed_form():
    # o = sigma(D) v1 + (1 - sigma(D)) v2 with D = scale * q.(k1 - k2)
    rng = np.random.default_rng(2)
    q, k, v = rand(rng, 1, 1, 5), rand(rng, 2, 1, 5), rand(rng, 2, 1, 5)
    scale = 0.7
    o = ao.attention_suffix(q, k, v, start=1, scale=scale)
    D = scale * float(q[0, 0] @ (k[0, 0] - k[1, 0]))
    s = 1.0 / (1.0 + math.exp(-D))
    np.testing.assert_allclose(o[0, 0], s * v[0, 0] + (1 - s) * v[1, 0], rtol=1e-13)


def test_future_keys_and_values_do_not_reach_a_query_and_its_own_do():
    rng = np.random.default_rng(3)
    start, n = 3, 5
    q, k, v = rand(rng, n, 2, 4), rand(rng, start + n, 2, 4), rand(rng, start + n, 2, 4)
    base = ao.attention_suffix(q, k, v, start, 0.5)
    for i in range(n):
        own = start + i                      # 0-based row of query i's own key
        k2, v2 = k.copy(), v.copy()
        k2[own + 1:] += 100.0                # a huge logit in the future must not leak
        v2[own + 1:] -= 50.0
        got = ao.attention_suffix(q, k2, v2, start, 0.5)
        np.testing.assert_array_equal(got[:i + 1], base[:i + 1])
        v3 = v.copy()
        v3[own] += 1.0                       # the query's own position is visible
        got = ao.attention_suffix(q, k, v3, start, 0.5)
        assert np.abs(got[i] - base[i]).max() > 1e-3
        assert np.array_equal(got[:i], base[:i])


def test_resuming_at_c_equals_the_rows_after_c_of_the_full_prefill():
    # the exact-reuse property the cache relies on
    rng = np.random.default_rng(4)
    N = 23
    q, k, v = rand(rng, N, 4, 8), rand(rng, N, 2, 8), rand(rng, N, 2, 8)
    full = ao.attention_suffix(q, k, v, 0, 0.35)
    for c in (1, 7, 22):
        part = ao.attention_suffix(q[c:], k, v, c, 0.35)
        np.testing.assert_allclose(part, full[c:], rtol=1e-13, atol=1e-15)


def test_brute_force_with_scalar_loops():
    rng = np.random.default_rng(5)
    start, n, H_q, H_kv, d = 2, 4, 4, 2, 3
    q, k, v = rand(rng, n, H_q, d), rand(rng, start + n, H_kv, d), rand(rng, start + n, H_kv, d)
    scale = 0.9
    o = ao.attention_suffix(q, k, v, start, scale)
    for i in range(n):
        for h in range(H_q):
            g = h // (H_q // H_kv)
            t = start + i + 1
            e = []
            for j in range(t):
                e.append(math.exp(scale * sum(q[i, h, x] * k[j, g, x] for x in range(d))))
            z = sum(e)
            for x in range(d):
                want = sum(e[j] * v[j, g, x] for j in range(t)) / z
                assert abs(o[i, h, x] - want) <= 1e-13 * max(1.0, abs(want))


def test_against_a_library_softmax_on_the_last_row():
    rng = np.random.default_rng(6)
    N, d = 40, 16
    q, k, v = rand(rng, N, 1, d), rand(rng, N, 1, d), rand(rng, N, 1, d)
    o = ao.attention_suffix(q[-1:], k, v, N - 1, 1.0 / math.sqrt(d))
    w = scipy_softmax((k[:, 0] @ q[-1, 0]) / math.sqrt(d))
    np.testing.assert_allclose(o[0, 0], w @ v[:, 0], rtol=1e-12)


def test_query_heads_read_the_key_value_head_of_their_group():
    rng = np.random.default_rng(7)
    n, H_q, H_kv, d = 3, 6, 3, 4
    q, k = rand(rng, n, H_q, d), rand(rng, n, H_kv, d)
    v = np.zeros((n, H_kv, d))
    for g in range(H_kv):
        v[:, g] = 10.0 * (g + 1)             # constant per kv head: a convex mix returns it
    o = ao.attention_suffix(q, k, v, 0, 1.0)
    for h in range(H_q):
        np.testing.assert_allclose(o[:, h], 10.0 * (h // 2 + 1), rtol=1e-13)


def test_a_common_shift_of_all_keys_changes_nothing_and_large_logits_stay_finite():
    rng = np.random.default_rng(8)
    n, d = 5, 4
    q, k, v = rand(rng, n, 1, d), rand(rng, n, 1, d), rand(rng, n, 1, d)
    base = ao.attention_suffix(q, k, v, 0, 1.0)
    shifted = ao.attention_suffix(q, k + rand(rng, 1, 1, d), v, 0, 1.0)
    np.testing.assert_allclose(shifted, base, rtol=1e-11)
    big = ao.attention_suffix(1e3 * q, 1e3 * k, v, 0, 1.0)   # logits ~1e6: exp would overflow unshifted
    assert np.isfinite(big).all()


def test_peaked_logits_select_the_best_visible_key():
    # orthogonal keys, query along key m: with a large scale the output is v_m once m is visible
    d = 8
    k = np.eye(d)[:, None, :] * 1.0                       # key j = e_j
    v = np.arange(d * 2, dtype=np.float64).reshape(d, 1, 2)
    q = np.tile(np.eye(d)[3][None, None, :], (d, 1, 1))   # every query asks for key 3 (position 4)
    o = ao.attention_suffix(q, k, v, 0, 200.0)
    for i in range(d):
        if i >= 3:
            np.testing.assert_allclose(o[i, 0], v[3, 0], atol=1e-12)
        else:                                             # key 3 is in the future: uniform over the visible ones
            np.testing.assert_allclose(o[i, 0], v[:i + 1, 0].mean(axis=0), rtol=1e-12)


def test_append_places_the_suffix_rows_and_nothing_else():
    rng = np.random.default_rng(9)
    kc, vc = rand(rng, 10, 2, 4), rand(rng, 10, 2, 4)
    kn, vn = rand(rng, 3, 2, 4), rand(rng, 3, 2, 4)
    k2, v2 = ao.append_kv(kc, vc, kn, vn, start=4)
    assert np.array_equal(k2[4:7], kn) and np.array_equal(v2[4:7], vn)
    assert np.array_equal(k2[:4], kc[:4]) and np.array_equal(k2[7:], kc[7:])
    assert np.array_equal(v2[:4], vc[:4]) and np.array_equal(v2[7:], vc[7:])
    with pytest.raises(AssertionError):
        ao.append_kv(kc, vc, kn, vn, start=8)


def test_output_gate_closed_forms():
    o = np.array([2.0, -4.0, 1.0])
    np.testing.assert_allclose(ao.output_gate(o, np.zeros(3)), o / 2, rtol=1e-15)
    np.testing.assert_allclose(ao.output_gate(o, np.full(3, 40.0)), o, rtol=1e-15)
    np.testing.assert_allclose(ao.output_gate(o, np.full(3, -40.0)), 0.0, atol=1e-15)
    g = np.array([0.3, -1.2, 2.0])
    np.testing.assert_allclose(ao.output_gate(o, g), o * 0.5 * (1 + np.tanh(g / 2)), rtol=1e-13)
