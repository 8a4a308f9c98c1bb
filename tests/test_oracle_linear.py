"""Pins for the projection oracle (Eq. 1: Q, K, V = X W): values worked by hand, one-hot weights that must select
columns of x (a transposed operand would select rows of the wrong thing or fail on the shapes), the identity, and
linearity.  None of them calls the same routine with the same formula."""
import numpy as np

import oracle


def _bf16(a):
    a = np.asarray(a, np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16)      # exact for the small integers and halves used here


def test_hand_worked_values():
    x = np.array([[1, 2, 3], [4, 5, 6]], np.float32)                       # M = 2, K = 3
    w = np.array([[1, 0, -1], [2, 1, 0], [0, 0, 1], [1, 1, 1]], np.float32)  # N = 4, K = 3
    want = np.array([[-2, 4, 3, 6], [-2, 13, 6, 15]], np.float64)
    assert np.array_equal(oracle.linear(x, w), want)
    assert np.array_equal(oracle.linear(_bf16(x), _bf16(w)), want)         # the same through bf16 storage


def test_one_hot_rows_select_columns_of_x():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 7)).astype(np.float32)
    sel = [6, 0, 3]
    w = np.zeros((3, 7), np.float32)
    for n, k in enumerate(sel):
        w[n, k] = 1.0
    assert np.array_equal(oracle.linear(x, w), x[:, sel].astype(np.float64))


def test_identity_and_linearity():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, 6)).astype(np.float32)
    assert np.array_equal(oracle.linear(x, np.eye(6, dtype=np.float32)), x.astype(np.float64))
    w1, w2 = (rng.integers(-3, 4, (5, 6)).astype(np.float32) for _ in range(2))
    a = oracle.linear(x, w1) + 2.0 * oracle.linear(x, w2)
    b = oracle.linear(x, w1 + 2.0 * w2)
    assert np.allclose(a, b, rtol=0, atol=1e-12)


def test_shapes_are_m_by_out_features():
    y = oracle.linear(np.zeros((3, 8), np.float32), np.zeros((5, 8), np.float32))
    assert y.shape == (3, 5) and y.dtype == np.float64
