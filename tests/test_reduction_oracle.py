"""Pins of the reduction / softmax oracle: closed forms, invariants, a library routine and exact rationals."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

from oracle import reduction as red


def test_sum_of_arithmetic_series_and_constants():
    n = 1000
    x = np.arange(1, n + 1, dtype=np.float64)[None, :].repeat(3, axis=0)
    assert red.reduce_rows(x, red.SUM).tolist() == [n * (n + 1) / 2] * 3  # Gauss
    assert red.reduce_rows(x, red.MEAN).tolist() == [(n + 1) / 2] * 3
    assert red.reduce_rows(x, red.MAX).tolist() == [float(n)] * 3
    x = np.full((2, 77), 0.1)
    assert red.reduce_rows(x, red.SUM)[0] == pytest.approx(7.7, rel=1e-15)


def test_sum_is_exact_where_naive_summation_is_not():
    # 1e16 + 1 - 1e16 loses the 1 in left-to-right double arithmetic; the exact sum is 1
    x = np.array([[1e16, 1.0, -1e16], [3.0, 1e-30, -3.0]])
    assert red.reduce_rows(x, red.SUM).tolist() == [1.0, 1e-30]
    rng = np.random.default_rng(5)
    v = rng.integers(-1000, 1000, size=(4, 50))
    assert red.reduce_rows(v / 7.0, red.SUM) == pytest.approx([float(Fraction(int(r.sum()), 7)) for r in v], rel=1e-15)


def test_max_picks_the_largest_and_not_the_largest_magnitude():
    x = np.array([[-5.0, -1.0, -3.0], [2.0, -9.0, 1.0]])
    assert red.reduce_rows(x, red.MAX).tolist() == [-1.0, 2.0]


def test_reduce_degenerate_shapes():
    assert red.reduce_rows(np.zeros((2, 0)), red.SUM).tolist() == [0.0, 0.0]
    assert red.reduce_rows(np.zeros((2, 0)), red.MAX).tolist() == [-np.inf, -np.inf]
    assert red.reduce_rows(np.zeros((0, 5)), red.SUM).shape == (0,)


def test_softmax_closed_forms():
    # constant row -> uniform; two entries -> logistic function of their difference
    assert red.softmax_rows(np.full((1, 8), 3.25))[0].tolist() == [0.125] * 8
    a, b = 0.3, -1.1
    y = red.softmax_rows(np.array([[a, b]]))[0]
    assert y[0] == pytest.approx(1.0 / (1.0 + np.exp(b - a)), rel=1e-15)
    assert y[1] == pytest.approx(1.0 / (1.0 + np.exp(a - b)), rel=1e-15)
    # log-ratios recover the input differences: y_i / y_j = exp(x_i - x_j)
    x = np.array([[0.5, -2.0, 1.5, 0.0]])
    y = red.softmax_rows(x)[0]
    for i in range(4):
        for j in range(4):
            assert np.log(y[i] / y[j]) == pytest.approx(x[0, i] - x[0, j], abs=1e-14)


def test_softmax_invariants_and_library():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((7, 33)) * 4
    y = red.softmax_rows(x)
    assert np.all(y > 0) and np.allclose(y.sum(axis=1), 1.0, rtol=0, atol=1e-15)
    assert np.allclose(red.softmax_rows(x + 123.0), y, rtol=1e-12, atol=0)  # shift invariance
    assert np.allclose(y, scipy.special.softmax(x, axis=1), rtol=1e-14, atol=0)
    assert np.array_equal(np.argsort(y, axis=1), np.argsort(x, axis=1))  # monotone
    # a plausible mistake -- normalising over the wrong axis -- is caught by the row sums above; another --
    # forgetting the max subtraction -- by the overflow case here
    big = np.array([[1000.0, 1000.0, -np.inf]])
    assert red.softmax_rows(big)[0].tolist() == [0.5, 0.5, 0.0]


def test_attention_reduces_to_known_cases():
    rng = np.random.default_rng(3)
    b, s, d = 2, 6, 4
    V = rng.standard_normal((b, s, d))
    # alpha = 0: uniform weights -> every output row is the mean of V's rows
    out = red.attention(rng.standard_normal((b, s, d)), rng.standard_normal((b, s, d)), V, 0.0)
    assert np.allclose(out, V.mean(axis=1, keepdims=True).repeat(s, axis=1), rtol=1e-13)
    # orthogonal one-hot keys with a huge scale: attention becomes a hard lookup of the matching value row
    Q = np.zeros((1, 4, 4))
    K = np.zeros((1, 4, 4))
    perm = [2, 0, 3, 1]
    for i in range(4):
        Q[0, i, i] = 1.0
        K[0, perm[i], i] = 1.0
    V = rng.standard_normal((1, 4, 4))
    out = red.attention(Q, K, V, 1e4)
    assert np.allclose(out[0], V[0][perm], rtol=1e-12)
    # against torch's own softmax/matmul in float64
    import torch
    Q, K, V = (rng.standard_normal((b, s, d)) for _ in range(3))
    ref = torch.softmax(0.5 * torch.from_numpy(Q) @ torch.from_numpy(K).transpose(1, 2), dim=-1) @ torch.from_numpy(V)
    assert np.allclose(red.attention(Q, K, V, 0.5), ref.numpy(), rtol=1e-12)
