"""Pins of the placement oracle (oracle/placement_oracle.py) against what the paper and the
mathematics fix: the closed form and worst case of Theorem 1, exhaustive search over all
checkpoint sets for tiny N, Table 1's tail-recompute column, the stability lemma, and a case
worked by hand.  CPU only."""
import itertools
import math

import numpy as np
import pytest

from oracle import placement_oracle as po


def thm1_closed_form(N, M):
    """Theorem 1: E[r] of a balanced set under uniform overlap, N + 1 = q K + rho, K = M + 1."""
    K = M + 1
    q, rho = divmod(N + 1, K)
    return ((K - rho) * q * (q - 1) / 2 + rho * q * (q + 1) / 2) / N


def brute_force(p, M):
    N = len(p)
    best = math.inf
    for m in range(0, M + 1):
        for C in itertools.combinations(range(1, N + 1), m):
            cost = 0.0
            for t in range(1, N + 1):
                l = max([0] + [c for c in C if c <= t])
                cost += p[t - 1] * (t - l)
            best = min(best, cost)
    return best


def test_hand_worked_case():
    # N = 4, p = (.1, .2, .3, .4), C = {3}: r(1..4) = 1, 2, 0, 1
    p = [0.1, 0.2, 0.3, 0.4]
    assert po.expected_recompute(p, [3]) == pytest.approx(0.1 * 1 + 0.2 * 2 + 0.0 + 0.4 * 1)
    assert po.no_cache_cost(p) == pytest.approx(3.0)
    assert po.savings(p, [3]) == pytest.approx(0.7)
    assert po.reduction(p, [3]) == pytest.approx(3.0 / 0.9)
    assert po.savings(p, []) == pytest.approx(0.0)
    assert [po.deepest([2, 3], t) for t in range(0, 5)] == [0, 0, 2, 3, 3]


@pytest.mark.parametrize("N,M", [(10, 1), (10, 3), (17, 4), (64, 7), (100, 9), (31, 31), (50, 0)])
def test_theorem1_closed_form_worst_case_and_dp_under_uniform_overlap(N, M):
    p = [1.0 / N] * N
    C = po.balanced(N, M)
    assert len(C) == M and all(1 <= c <= N for c in C) and sorted(set(C)) == C
    gaps = np.diff([0] + C + [N + 1])
    assert gaps.max() - gaps.min() <= 1                           # balanced in the paper's sense
    assert po.expected_recompute(p, C) == pytest.approx(thm1_closed_form(N, M), abs=1e-12)
    worst = max(t - po.deepest(C, t) for t in range(1, N + 1))
    assert worst == math.ceil((N + 1) / (M + 1)) - 1
    cost, pos = po.dp_optimal(p, M)
    assert cost == pytest.approx(thm1_closed_form(N, M), abs=1e-12)  # balanced is optimal, so the DP ties it
    assert po.expected_recompute(p, pos) == pytest.approx(cost, abs=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_dp_equals_exhaustive_search_on_tiny_inputs(seed):
    rng = np.random.default_rng(seed)
    N = int(rng.integers(3, 11))
    M = int(rng.integers(0, 4))
    p = rng.random(N)
    if seed % 2:
        p[rng.integers(0, N, size=N // 2)] = 0.0                  # zero-mass depths: ties in the hull
    p = list(p / max(p.sum(), 1e-300)) if p.sum() > 0 else [1.0 / N] * N
    cost, pos = po.dp_optimal(p, M)
    assert len(pos) <= M and sorted(set(pos)) == pos and all(1 <= c <= N for c in pos)
    assert cost == pytest.approx(brute_force(p, M), abs=1e-12)
    assert po.expected_recompute(p, pos) == pytest.approx(cost, abs=1e-12)


def test_point_mass_is_served_exactly():
    N = 40
    p = [0.0] * N
    p[26] = 1.0                                                    # all overlap at depth 27
    cost, pos = po.dp_optimal(p, 1)
    assert cost == 0.0 and pos == [27]


@pytest.mark.parametrize("L,B,M", [(1000, 128, 5), (8192, 128, 16), (777, 64, 3)])
def test_table1_positions_and_tail_recompute(L, B, M):
    assert L - po.deepest(po.block(L, B), L) == L % B
    s = math.isqrt(L)
    assert L - po.deepest(po.sqrt_spaced(L), L) == L % s
    worst = max(t - po.deepest(po.balanced(L, M), t) for t in range(1, L + 1))
    assert worst == math.ceil((L + 1) / (M + 1)) - 1
    lg = po.logarithmic(L, B, M)
    assert lg[0] == B and all(b - a == 2 * (a - z) for z, a, b in zip([0] + lg, lg, lg[1:]))   # gaps double
    assert lg[-1] <= L and len(lg) <= M


def test_clip_to_blocks():
    assert po.clip_to_blocks([130, 255, 256, 60, 1000], 128) == [128, 256, 896]
    assert po.clip_to_blocks([5, 64, 127], 128) == []


@pytest.mark.parametrize("seed", range(4))
def test_stability_lemma_and_dp_dominates_baselines(seed):
    rng = np.random.default_rng(100 + seed)
    N, M = 60, 5
    p = rng.random(N) ** 3; p /= p.sum()
    q = rng.random(N); q /= q.sum()
    C = sorted(rng.choice(np.arange(1, N + 1), size=M, replace=False).tolist())
    lhs = abs(po.expected_recompute(p, C) - po.expected_recompute(q, C))
    assert lhs <= N * np.abs(p - q).sum() + 1e-12                 # |E_p r - E_q r| <= N ||p - q||_1
    cost, pos = po.dp_optimal(p, M)
    for base in (po.balanced(N, M), po.block(N, 12)[:M], po.sqrt_spaced(N)[:M], po.logarithmic(N, 1, M), C):
        assert cost <= po.expected_recompute(p, base) + 1e-12
    assert cost <= po.dp_optimal(p, M - 1)[0] + 1e-12             # a larger budget never hurts
