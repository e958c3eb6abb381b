"""The error measure of the parity tests (CPU): per (request, layer, value head), so that a head whose outputs are
small is not judged against the largest head of the call."""
import numpy as np

from tests.harness import max_norm_err, worst_head_err, worst_state_err


def test_small_head_is_judged_against_itself():
    rng = np.random.default_rng(0)
    ref = rng.standard_normal((2, 30, 3, 8))
    ref[1, 10:30, 2] *= 1e-3                 # request 1 (tokens 10..29), layer 1, head 2: small outputs
    x = ref.copy()
    x[1, 17, 2, 5] += 1e-5                   # an error of 1 % of that head's scale
    cu = [0, 10, 30]
    err, where = worst_head_err(x, ref, cu)
    assert where == (1, 1, 2)
    den = np.abs(ref[1, 10:30, 2]).max()
    assert np.isclose(err, 1e-5 / den)
    assert max_norm_err(x, ref) < err / 100  # the whole-call reading would have let it pass


def test_empty_requests_and_exact_match():
    ref = np.ones((1, 4, 2, 3))
    assert worst_head_err(ref, ref, [0, 0, 4, 4]) == (0.0, None)


def test_state_measure_is_per_head():
    ref = np.ones((1, 2, 4, 4))
    ref[0, 1] *= 1e-4
    x = ref.copy()
    x[0, 1, 2, 3] += 1e-6
    assert np.isclose(worst_state_err(x, ref), 1e-2)
