"""Oracle of the checkpoint placement layer.  TEST INFRASTRUCTURE ONLY.

Only tests/ may import this module.  It shares no code with the library: plain Python and
numpy, fp64, every function the definition written out.

What it follows (paper sections, in its notation: N prefix length, M budget, p_t mass of
overlap depth t = 1..N, checkpoint set C = {c_1 < ... < c_M} in [1, N]):
  Sec. 3            deepest reusable checkpoint l(t; C) = max({0} U {c in C : c <= t}),
                    recomputation r = t - l, no-cache work R_nc = sum p_t t,
                    Savings = 1 - E[r] / R_nc, Reduction = R_nc / E[r]
  Table 1           Balanced floor(i (L+1) / (M+1)), Block B, 2B, ..., sqrt(L)-spaced
  Sec. 5 baselines  Logarithmic: gap sizes growing exponentially from the beginning of the
                    prefix (base and unit are not given; reading: gaps unit, 2 unit, 4 unit,
                    ..., i.e. positions unit (2^i - 1), at most M of them)
  Sec. 5            clipping of every position to block boundaries (reading: floor to a
                    multiple of B; zeros and duplicates dropped)
  Theorem 2         dp[0, j] = sum_{t<=j} p_t t,
                    dp[m, j] = min_{1<=s<=j} dp[m-1, s-1] + w(s, j), w(s, j) = sum_{t=s..j} p_t (t - s)
                    (dp[m, 0] = 0: no depth to serve costs nothing, so fewer than m
                    checkpoints may end up placed)
The dynamic program here is the recurrence evaluated as printed, O(N^2 M), with explicit
sums: no prefix-sum rewriting, no hull.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np


def deepest(pos: Sequence[int], t: int) -> int:
    """l(t; C): the largest checkpoint position <= t, or 0."""
    best = 0
    for c in pos:
        if c <= t and c > best:
            best = c
    return best


def expected_recompute(p: Sequence[float], pos: Sequence[int]) -> float:
    """E[r(T; C)] = sum_t p_t (t - l(t; C)), p[t-1] = p_t (weights need not sum to one)."""
    return float(sum(float(p[t - 1]) * (t - deepest(pos, t)) for t in range(1, len(p) + 1)))


def no_cache_cost(p: Sequence[float]) -> float:
    return float(sum(float(p[t - 1]) * t for t in range(1, len(p) + 1)))


def savings(p, pos) -> float:
    return 1.0 - expected_recompute(p, pos) / no_cache_cost(p)


def reduction(p, pos) -> float:
    return no_cache_cost(p) / expected_recompute(p, pos)


def balanced(N: int, M: int) -> List[int]:
    return [(i * (N + 1)) // (M + 1) for i in range(1, M + 1)]


def block(N: int, B: int) -> List[int]:
    return [B * i for i in range(1, N // B + 1)]


def sqrt_spaced(N: int) -> List[int]:
    s = math.isqrt(N)
    return [s * i for i in range(1, N // s + 1)]


def logarithmic(N: int, unit: int, M: int) -> List[int]:
    out, i = [], 1
    while len(out) < M and unit * (2 ** i - 1) <= N:
        out.append(unit * (2 ** i - 1))
        i += 1
    return out


def clip_to_blocks(pos: Sequence[int], B: int) -> List[int]:
    out: List[int] = []
    for c in sorted(pos):
        c = (c // B) * B
        if c > 0 and (not out or out[-1] != c):
            out.append(c)
    return out


def dp_optimal(p: Sequence[float], M: int) -> Tuple[float, List[int]]:
    """Minimum expected recomputation with at most M checkpoints and one optimal set."""
    N = len(p)
    w = np.zeros((N + 2, N + 1))
    for s in range(1, N + 1):
        acc = 0.0
        for j in range(s, N + 1):
            acc += float(p[j - 1]) * (j - s)
            w[s, j] = acc
    dp = np.zeros((M + 1, N + 1))
    arg = np.zeros((M + 1, N + 1), dtype=np.int64)
    for j in range(1, N + 1):
        dp[0, j] = dp[0, j - 1] + float(p[j - 1]) * j
    for m in range(1, M + 1):
        for j in range(1, N + 1):
            best, best_s = math.inf, 0
            for s in range(1, j + 1):
                v = dp[m - 1, s - 1] + w[s, j]
                if v < best:
                    best, best_s = v, s
            dp[m, j], arg[m, j] = best, best_s
    pos, j, m = [], N, M
    while m > 0 and j > 0:
        s = int(arg[m, j])
        pos.append(s)
        j, m = s - 1, m - 1
    return float(dp[M, N]), sorted(pos)
