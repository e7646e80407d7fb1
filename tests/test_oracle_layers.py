"""Pins for the oracle's layer mathematics: brute-force loops, closed forms and
central finite differences on tiny nets."""
import math

import numpy as np
import pytest

from oracle import layers as L


def test_dense_forward_brute_force():
    rng = np.random.default_rng(1)
    x, W, b = rng.standard_normal((3, 5)), rng.standard_normal((4, 5)), rng.standard_normal(4)
    z = L.dense_forward(x, W, b)
    for i in range(3):
        for o in range(4):
            ref = b[o] + sum(x[i, k] * W[o, k] for k in range(5))
            assert abs(z[i, o] - ref) < 1e-13


def test_dense_backward_brute_force():
    rng = np.random.default_rng(2)
    dz, x, W = rng.standard_normal((3, 4)), rng.standard_normal((3, 5)), rng.standard_normal((4, 5))
    dW, db, dx = L.dense_backward(dz, x, W)
    for o in range(4):
        assert abs(db[o] - sum(dz[i, o] for i in range(3))) < 1e-13
        for k in range(5):
            assert abs(dW[o, k] - sum(dz[i, o] * x[i, k] for i in range(3))) < 1e-13
    for i in range(3):
        for k in range(5):
            assert abs(dx[i, k] - sum(dz[i, o] * W[o, k] for o in range(4))) < 1e-13


def test_activation_values():
    z = np.array([-2.0, -0.5, 0.0, 0.5, 2.0])
    assert np.array_equal(L.act_forward(z, "relu"), [0, 0, 0, 0.5, 2.0])
    assert np.array_equal(L.act_derivative(z, "relu"), [0, 0, 0, 1, 1])
    # GELU(z) = z * Phi(z) with the standard normal CDF, written with math.erfc
    ref = [v * 0.5 * math.erfc(-v / math.sqrt(2)) for v in z]
    assert np.allclose(L.act_forward(z, "gelu"), ref, rtol=0, atol=1e-15)
    # known values: GELU(0)=0, GELU'(0)=1/2, GELU(z) -> z for large z
    assert L.act_forward(np.array([0.0]), "gelu")[0] == 0.0
    assert L.act_derivative(np.array([0.0]), "gelu")[0] == 0.5
    assert abs(L.act_forward(np.array([10.0]), "gelu")[0] - 10.0) < 1e-12


@pytest.mark.parametrize("act", ["gelu", "relu"])
def test_activation_derivative_finite_difference(act):
    z = np.array([-1.7, -0.3, 0.2, 0.9, 2.4])
    h = 1e-6
    fd = (L.act_forward(z + h, act) - L.act_forward(z - h, act)) / (2 * h)
    assert np.allclose(L.act_derivative(z, act), fd, rtol=0, atol=1e-8)


def test_softmax_ce_closed_forms():
    # uniform logits: loss = log(C); gradient = (1/C - onehot)/denom
    C, rows = 7, 3
    logits = np.zeros((rows, C))
    labels = np.array([0, 3, 6])
    loss, d = L.softmax_cross_entropy(logits, labels, denom=rows)
    assert abs(loss - math.log(C)) < 1e-14
    ref = np.full((rows, C), 1.0 / C)
    ref[np.arange(rows), labels] -= 1.0
    assert np.allclose(d, ref / rows, rtol=0, atol=1e-15)
    # shift invariance and rows of the gradient summing to zero
    rng = np.random.default_rng(3)
    lg = rng.standard_normal((4, 5)) * 3
    lb = np.array([1, 0, 4, 2])
    l1, d1 = L.softmax_cross_entropy(lg, lb, 4)
    l2, d2 = L.softmax_cross_entropy(lg + 100.0, lb, 4)
    assert abs(l1 - l2) < 1e-12 and np.allclose(d1, d2, atol=1e-14)
    assert np.allclose(d1.sum(axis=1), 0, atol=1e-15)
    # brute force
    ref_loss = 0.0
    for r in range(4):
        ref_loss -= math.log(math.exp(lg[r, lb[r]]) / sum(math.exp(v) for v in lg[r]))
    assert abs(l1 - ref_loss / 4) < 1e-12


def test_softmax_ce_gradient_finite_difference():
    rng = np.random.default_rng(4)
    lg = rng.standard_normal((3, 6))
    lb = np.array([5, 0, 2])
    _, d = L.softmax_cross_entropy(lg, lb, 12)
    h = 1e-6
    for r in range(3):
        for c in range(6):
            p, m = lg.copy(), lg.copy()
            p[r, c] += h
            m[r, c] -= h
            fd = (L.softmax_cross_entropy(p, lb, 12)[0] - L.softmax_cross_entropy(m, lb, 12)[0]) / (2 * h)
            assert abs(d[r, c] - fd) < 1e-9
