"""Pins of the layer oracle (oracle/layer_oracle.py) against what the mathematics and library
routines fix: the convolution against numpy's and torch's own convolutions and its impulse
response, resume == full replay for the convolution state, closed forms of SiLU, the gates and
the two normalisations.  Each pin is chosen so that a plausible slip (reversed taps, an
off-by-one state row, eps outside the root, mean instead of sum) fails it.
"""
import numpy as np
import pytest

from oracle import layer_oracle as lo


def rng_for(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------- convolution
@pytest.mark.parametrize("K", [2, 3, 4])
def test_conv_is_the_library_convolution_with_the_last_tap_on_the_current_token(K):
    rng = rng_for(10 + K)
    T, C = 23, 5
    x, w, b = rng.standard_normal((T, C)), rng.standard_normal((C, K)), rng.standard_normal(C)
    y = lo.short_conv_pre(x, w, b, None)
    for c in range(C):
        ref = np.convolve(x[:, c], w[c, ::-1])[:T] + b[c]        # convolution with the flipped kernel
        assert np.allclose(y[:, c], ref, rtol=0, atol=1e-13)
    import torch
    xt = torch.from_numpy(x.T.copy())[None]                      # [1][C][T]
    ref_t = torch.nn.functional.conv1d(xt, torch.from_numpy(w)[:, None, :], torch.from_numpy(b), padding=K - 1, groups=C)
    assert np.allclose(y, ref_t[0, :, :T].numpy().T, rtol=0, atol=1e-13)


def test_conv_impulse_response_reads_the_taps_backwards_in_time():
    K, C, T, t0 = 4, 3, 12, 5
    w = np.arange(1.0, 1.0 + C * K).reshape(C, K)
    x = np.zeros((T, C))
    x[t0, 1] = 1.0
    y = lo.short_conv_pre(x, w, None, None)
    for j in range(K):
        assert y[t0 + j, 1] == w[1, K - 1 - j]      # tap K-1 acts at once, tap 0 K-1 tokens later
    assert np.count_nonzero(y) == K


def test_conv_hand_worked_case():
    # one channel, K = 3, w = (1, 10, 100), x = 1, 2, 3 after a state (7, 8): y_t = x_{t-2} + 10 x_{t-1} + 100 x_t
    y = lo.short_conv_pre(np.array([[1.0], [2.0], [3.0]]), np.array([[1.0, 10.0, 100.0]]), None, np.array([[7.0], [8.0]]))
    assert y[:, 0].tolist() == [7 + 80 + 100, 8 + 10 + 200, 1 + 20 + 300]


@pytest.mark.parametrize("p", [0, 1, 2, 3, 7, 19, 20])
def test_conv_resume_equals_full_replay_bitwise(p):
    """Splitting a sequence at p and continuing from the stored rows changes no output bit."""
    rng = rng_for(77)
    K, T, C = 4, 20, 6
    x, w, b = rng.standard_normal((T, C)), rng.standard_normal((C, K)), rng.standard_normal(C)
    full = lo.short_conv_pre(x, w, b, None)
    st = lo.conv_state_after(x, None, K, p)
    assert st.shape == (K - 1, C)
    for i in range(K - 1):                                      # rows x[p-3], x[p-2], x[p-1]; zeros before the start
        s = p - (K - 1) + i
        assert np.array_equal(st[i], x[s] if s >= 0 else np.zeros(C))
    resumed = lo.short_conv_pre(x[p:], w, b, st)
    assert np.array_equal(resumed, full[p:])
    # chaining: the state a resumed run stores further on is the one the full run stores there
    for p2 in range(p, T + 1):
        assert np.array_equal(lo.conv_state_after(x[p:], st, K, p2 - p), lo.conv_state_after(x, None, K, p2))


def test_conv_wrong_state_is_detected_only_in_the_first_taps():
    """A perturbed state row changes exactly the first K-1 outputs: the window the parity tests must look at."""
    rng = rng_for(5)
    K, T, C = 4, 10, 2
    x, w = rng.standard_normal((T, C)), rng.standard_normal((C, K))
    st = rng.standard_normal((K - 1, C))
    bad = st.copy()
    bad[0] += 1.0                                               # the oldest row reaches only the first output
    d = lo.short_conv_pre(x, w, None, st) - lo.short_conv_pre(x, w, None, bad)
    assert np.all(d[0] != 0) and np.all(d[1:] == 0)
    bad = st.copy()
    bad[K - 2] += 1.0                                           # the newest row reaches K-1 outputs
    d = lo.short_conv_pre(x, w, None, st) - lo.short_conv_pre(x, w, None, bad)
    assert np.all(d[:K - 1] != 0) and np.all(d[K - 1:] == 0)


# ----------------------------------------------------------------------------- activations, gates
def test_silu_closed_forms():
    x = np.linspace(-20, 20, 401)
    assert lo.silu(0.0) == 0.0
    assert np.allclose(lo.silu(x) - lo.silu(-x), x, rtol=0, atol=1e-12)      # x s(x) - (-x)(1 - s(x)) = x
    assert abs(lo.silu(40.0) - 40.0) < 1e-12 and abs(lo.silu(-40.0)) < 1e-12
    xm = 1.2784645427610738                                                  # the minimiser x* = -xm solves 1 + x (1 - s(x)) = 0,
    assert abs(lo.silu(-xm) - (-0.2784645427610738)) < 1e-12                 # hence s(x*) = 1 + 1/x* and the minimum is x* + 1
    assert np.all(lo.silu(x) >= lo.silu(-xm) - 1e-15)


def test_gates_closed_forms():
    rng = rng_for(3)
    a, b = rng.standard_normal((50, 4)) * 3, rng.standard_normal((50, 4)) * 3
    zero = np.zeros(4)
    beta, gate = lo.gates(a, b, zero, zero)
    assert np.allclose(gate, 1.0 / (1.0 + np.exp(a)), rtol=1e-13, atol=0)    # exp(-softplus(a)) = sigmoid(-a)
    assert np.allclose(beta + lo.gates(a, -b, zero, zero)[0], 1.0, rtol=0, atol=1e-15)
    assert np.allclose(beta, 0.5 * (1.0 + np.tanh(0.5 * b)), rtol=1e-10, atol=0)     # cancellation near -1
    dt = rng.standard_normal(4)
    assert np.allclose(lo.gates(a, b, zero, dt)[1], lo.gates(a + dt[None, :], b, zero, zero)[1], rtol=1e-15, atol=0)
    A_log = rng.standard_normal(4)
    assert np.allclose(lo.gates(a, b, A_log, dt)[1], lo.gates(a, b, zero, dt)[1] ** np.exp(A_log)[None, :], rtol=1e-12, atol=0)
    assert np.all((gate > 0) & (gate < 1)) and np.all((beta > 0) & (beta < 1))
    big = lo.gates(np.full((1, 4), 50.0), b[:1], zero, zero)[1]
    assert np.allclose(big, np.exp(-50.0), rtol=1e-12, atol=0)               # softplus(x) -> x


# ----------------------------------------------------------------------------- normalisations
def test_l2norm_closed_forms():
    assert np.allclose(lo.l2norm(np.array([3.0, 4.0]), 0.0), [0.6, 0.8], rtol=0, atol=1e-16)
    assert np.allclose(lo.l2norm(np.array([3.0, 4.0]), 11.0), [0.5, 2.0 / 3.0], rtol=0, atol=1e-16)   # eps under the root: sqrt(36)
    x = rng_for(1).standard_normal((7, 3, 16))
    y = lo.l2norm(x, 0.0)
    assert np.allclose((y * y).sum(-1), 1.0, rtol=0, atol=1e-14)
    assert np.allclose(lo.l2norm(5.0 * x, 0.0), y, rtol=0, atol=1e-15)
    assert np.array_equal(lo.l2norm(x, 1e-6)[2, 1], lo.l2norm(x[2, 1], 1e-6))                          # per head, not per token


def test_output_norm_gate_closed_forms():
    rng = rng_for(2)
    T, H, d = 5, 3, 8
    o, z, w = rng.standard_normal((T, H, d)), rng.standard_normal((T, H, d)), rng.standard_normal(d)
    y = lo.output_norm_gate(o, z, w, 0.0)
    assert np.allclose(((y / (w * lo.silu(z))) ** 2).mean(-1), 1.0, rtol=0, atol=1e-12)                # unit mean square
    assert np.allclose(lo.output_norm_gate(7.0 * o, z, w, 0.0), y, rtol=0, atol=1e-14)
    assert np.all(lo.output_norm_gate(o, np.zeros_like(z), w, 1e-5) == 0.0)
    c = np.full((1, 1, d), -2.5)
    assert np.allclose(lo.output_norm_gate(c, z[:1, :1], np.ones(d), 0.0), -lo.silu(z[:1, :1]), rtol=0, atol=1e-15)
    # eps under the root, on the MEAN square: o = (2, 2, 2, 2), eps = 5 -> 2 / sqrt(4 + 5)
    y1 = lo.output_norm_gate(np.full((1, 1, 4), 2.0), np.full((1, 1, 4), 40.0), np.ones(4), 5.0)
    assert np.allclose(y1, 2.0 / 3.0 * 40.0, rtol=1e-12, atol=0)
    import torch
    ref = torch.nn.functional.rms_norm(torch.from_numpy(o), (d,), torch.from_numpy(w), 1e-5) * torch.nn.functional.silu(torch.from_numpy(z))
    assert np.allclose(lo.output_norm_gate(o, z, w, 1e-5), ref.numpy(), rtol=1e-13, atol=1e-14)


# ----------------------------------------------------------------------------- the packed call
def test_layer_inputs_packs_requests_and_emits_states_at_absolute_positions():
    rng = rng_for(9)
    H_qk, H_v, d_k, d_v, K = 1, 2, 4, 4, 4
    C = 2 * H_qk * d_k + H_v * d_v
    N = 12
    x = rng.standard_normal((N, C))
    w, b = rng.standard_normal((C, K)), rng.standard_normal(C)
    a_pre, b_pre = rng.standard_normal((N, H_v)), rng.standard_normal((N, H_v))
    A_log, dt = rng.standard_normal(H_v), rng.standard_normal(H_v)
    # full run: one request from position 0, states at 2, 5, 12
    full = lo.layer_inputs(x, w, b, a_pre, b_pre, A_log, dt, H_qk, H_v, d_k, d_v, [0, N], [0], [-1], None, [0, 3], [2, 5, 12], 1e-6)
    assert np.array_equal(full[5][0], np.vstack([np.zeros((1, C)), x[0:2]]))
    assert np.array_equal(full[5][1], x[2:5]) and np.array_equal(full[5][2], x[9:12])
    # two resumed requests packed: from 5 (slot 1) and from 2 (slot 0), rows of the same prefix
    pool = full[5]
    xs = np.vstack([x[5:], x[2:]])
    res = lo.layer_inputs(xs, w, b, np.vstack([a_pre[5:], a_pre[2:]]), np.vstack([b_pre[5:], b_pre[2:]]), A_log, dt, H_qk, H_v, d_k, d_v,
                          [0, N - 5, 2 * N - 7], [5, 2], [1, 0], pool, [0, 1, 3], [12, 5, 12], 1e-6)
    for i in range(5):
        assert np.array_equal(res[i][:N - 5], full[i][5:]) and np.array_equal(res[i][N - 5:], full[i][2:])
    assert np.array_equal(res[5][0], pool[2]) and np.array_equal(res[5][1], pool[1]) and np.array_equal(res[5][2], pool[2])
    # unit-norm q and k per head, v untouched by the normalisation
    assert np.allclose((full[0] ** 2).sum(-1), 1.0, atol=1e-5) and np.allclose((full[1] ** 2).sum(-1), 1.0, atol=1e-5)
    pre = lo.short_conv_pre(x, w, b, None)
    assert np.allclose(full[2].reshape(N, -1), lo.silu(pre[:, 2 * H_qk * d_k:]), rtol=0, atol=1e-15)
