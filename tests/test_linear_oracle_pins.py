"""Pins of the projection oracle (CPU): the definition against a hand-worked case, textbook special cases and its own
two forms."""
import numpy as np

from oracle import linear_oracle as lo
from paper_2605_05219_amd import workloads as wl


def test_hand_worked_case():
    # y = x w^T + b with w stored [out][in]:  x = [[1, 2, 3], [0, -1, 4]], w = [[1, 0, 2], [-1, 1, 0.5]], b = [10, 20]
    x = np.array([[1, 2, 3], [0, -1, 4]], np.float32)
    w = np.array([[1, 0, 2], [-1, 1, 0.5]], np.float32)
    b = np.array([10, 20], np.float32)
    want = np.array([[1 * 1 + 3 * 2 + 10, -1 + 2 + 1.5 + 20], [8 + 10, -1 + 2 + 20]], np.float64)
    assert np.array_equal(lo.linear_loops(x, w, b), want)
    assert np.array_equal(lo.linear(x, w, b), want)


def test_identity_permutation_and_bias_alone():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7)).astype(np.float32)
    assert np.array_equal(lo.linear(x, np.eye(7, dtype=np.float32)), x.astype(np.float64))
    perm = rng.permutation(7)
    w = np.eye(7, dtype=np.float32)[perm]              # row n of w picks input perm[n]
    assert np.array_equal(lo.linear(x, w), x.astype(np.float64)[:, perm])
    b = rng.standard_normal(3).astype(np.float32)
    assert np.array_equal(lo.linear(x, np.zeros((3, 7), np.float32), b), np.broadcast_to(b.astype(np.float64), (5, 3)))


def test_storage_is_out_by_in_not_transposed():
    x = np.array([[1.0, 2.0]], np.float32)
    w = np.array([[3.0, 4.0], [5.0, 6.0], [7.0, 8.0]], np.float32)      # three outputs, two inputs
    assert lo.linear(x, w).shape == (1, 3)
    assert np.array_equal(lo.linear(x, w), [[11.0, 17.0, 23.0]])


def test_loops_equal_matrix_product_and_linearity():
    rng = np.random.default_rng(1)
    x = wl.f32_to_bf16_bits(rng.standard_normal((9, 33)).astype(np.float32))
    x2 = wl.f32_to_bf16_bits(rng.standard_normal((9, 33)).astype(np.float32))
    w = wl.f32_to_bf16_bits(rng.standard_normal((13, 33)).astype(np.float32))
    b = rng.standard_normal(13).astype(np.float32)
    a, c = lo.linear_loops(x, w, b), lo.linear(x, w, b)
    assert np.abs(a - c).max() <= 1e-13 * np.abs(a).max()
    # linear in x (fp64 on exactly widened inputs): f(x) + f(x2) - f(0) = f(x + x2)
    xs = wl.to_f32(x).astype(np.float64) + wl.to_f32(x2).astype(np.float64)
    lhs = lo.linear(x, w, b) + lo.linear(x2, w, b) - b.astype(np.float64)[None, :]
    assert np.abs(lhs - lo.linear(xs, w, b)).max() <= 1e-12 * np.abs(lhs).max()


def test_bf16_bits_are_widened_exactly():
    bits = np.array([[0x3F80, 0xC000, 0x0001]], np.uint16)            # 1.0, -2.0, the smallest bf16 denormal
    w = np.array([[0x3F80, 0x3F80, 0x3F80]], np.uint16)
    want = 1.0 - 2.0 + float(np.array([0x0001 << 16], np.uint32).view(np.float32)[0])
    assert lo.linear(bits, w)[0, 0] == want
