"""Pins for the oracle's convolution and pooling: brute-force loops, reduction of a 1x1
convolution to a dense layer, finite differences through a conv/pool/conv stage, pooling ties."""
import numpy as np
import pytest

from oracle import layers as L
from oracle.stage import Stage
from synth_inputs.workloads import Conv2d, MaxPool2


def _brute_conv(x, W, b, stride, pad):
    B, H, Wd, Cin = x.shape
    Cout, kh, kw, _ = W.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (Wd + 2 * pad - kw) // stride + 1
    z = np.zeros((B, Ho, Wo, Cout))
    for n in range(B):
        for oh in range(Ho):
            for ow in range(Wo):
                for o in range(Cout):
                    s = b[o]
                    for i in range(kh):
                        for j in range(kw):
                            ih, iw = oh * stride + i - pad, ow * stride + j - pad
                            if 0 <= ih < H and 0 <= iw < Wd:
                                for c in range(Cin):
                                    s += x[n, ih, iw, c] * W[o, i, j, c]
                    z[n, oh, ow, o] = s
    return z


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 1, 3), (1, 0, 1), (2, 3, 7)])
def test_conv_forward_brute_force(stride, pad, k):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 7, 6, 3))
    W = rng.standard_normal((4, k, k, 3))
    b = rng.standard_normal(4)
    assert np.allclose(L.conv2d_forward(x, W, b, stride, pad), _brute_conv(x, W, b, stride, pad), atol=1e-12)


def test_conv_backward_brute_force():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 5, 4, 3))
    W = rng.standard_normal((4, 3, 3, 3))
    dz = rng.standard_normal((2, 5, 4, 4))
    dW, db, dx = L.conv2d_backward(dz, x, W, 1, 1)
    rW, rx = np.zeros_like(W), np.zeros_like(x)
    for n in range(2):
        for oh in range(5):
            for ow in range(4):
                for o in range(4):
                    for i in range(3):
                        for j in range(3):
                            ih, iw = oh + i - 1, ow + j - 1
                            if 0 <= ih < 5 and 0 <= iw < 4:
                                for c in range(3):
                                    rW[o, i, j, c] += dz[n, oh, ow, o] * x[n, ih, iw, c]
                                    rx[n, ih, iw, c] += dz[n, oh, ow, o] * W[o, i, j, c]
    assert np.allclose(dW, rW, atol=1e-12) and np.allclose(dx, rx, atol=1e-12)
    assert np.allclose(db, dz.sum(axis=(0, 1, 2)), atol=1e-12)


def test_one_by_one_conv_is_a_dense_layer_on_pixels():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 3, 3, 5))
    W = rng.standard_normal((4, 1, 1, 5))
    b = rng.standard_normal(4)
    z = L.conv2d_forward(x, W, b, 1, 0)
    assert np.allclose(z.reshape(-1, 4), L.dense_forward(x.reshape(-1, 5), W[:, 0, 0, :], b), atol=1e-13)
    dz = rng.standard_normal(z.shape)
    dW, db, dx = L.conv2d_backward(dz, x, W, 1, 0)
    rW, rb, rx = L.dense_backward(dz.reshape(-1, 4), x.reshape(-1, 5), W[:, 0, 0, :])
    assert np.allclose(dW[:, 0, 0, :], rW) and np.allclose(db, rb) and np.allclose(dx.reshape(-1, 5), rx)


def test_maxpool_values_ties_and_backward():
    x = np.zeros((1, 2, 4, 1))
    x[0, :, :, 0] = [[1, 3, 5, 5],
                     [3, 2, 5, 4]]
    y, idx = L.maxpool2_forward(x)
    assert y[0, 0, :, 0].tolist() == [3, 5]
    assert idx[0, 0, :, 0].tolist() == [1, 0]           # first maximum in row-major window order
    dx = L.maxpool2_backward(np.array([[[[10.0], [20.0]]]]), idx, x.shape)
    assert dx[0, :, :, 0].tolist() == [[0, 10, 20, 0], [0, 0, 0, 0]]
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 4, 6, 3))
    y, idx = L.maxpool2_forward(x)
    for n in range(2):
        for i in range(2):
            for j in range(3):
                for c in range(3):
                    assert y[n, i, j, c] == x[n, 2 * i:2 * i + 2, 2 * j:2 * j + 2, c].max()
    dy = rng.standard_normal(y.shape)
    dx = L.maxpool2_backward(dy, idx, x.shape)
    assert np.isclose(dx.sum(), dy.sum()) and np.count_nonzero(dx) == dy.size


def test_conv_pool_stage_gradients_match_finite_differences():
    specs = (Conv2d(2, 3, 4, 4, "gelu"), MaxPool2(3, 4, 4), Conv2d(3, 2, 2, 2, "gelu"))
    rng = np.random.default_rng(5)
    params = [rng.standard_normal((3, 3, 3, 2)) * 0.4, rng.standard_normal(3) * 0.1,
              rng.standard_normal((2, 3, 3, 3)) * 0.4, rng.standard_normal(2) * 0.1]
    x = rng.standard_normal((4, 4, 4, 2))
    target = rng.standard_normal((4, 2, 2, 2))

    def loss_of(plist, xin):
        st = Stage(specs, plist, policy="eq1", lam=0.1, lr=0.0, momentum=0.0, n=2)
        out = np.concatenate([st.forward(0, ub, xin[ub * 2:(ub + 1) * 2]) for ub in range(2)])
        return 0.5 * np.sum((out - target) ** 2), out, st

    loss, out, st = loss_of(params, x)
    dx = st.backward(0, out - target)
    h = 1e-6
    for pi, p in enumerate(params):
        for idx in list(np.ndindex(p.shape))[::3]:
            hi = [q.copy() for q in params]
            lo = [q.copy() for q in params]
            hi[pi][idx] += h
            lo[pi][idx] -= h
            fd = (loss_of(hi, x)[0] - loss_of(lo, x)[0]) / (2 * h)
            assert abs(st.g[pi][idx] - fd) < 1e-6, (pi, idx)
    for idx in list(np.ndindex(x.shape))[::5]:
        hi, lo = x.copy(), x.copy()
        hi[idx] += h
        lo[idx] -= h
        fd = (loss_of(params, hi)[0] - loss_of(params, lo)[0]) / (2 * h)
        assert abs(dx[idx] - fd) < 1e-6
