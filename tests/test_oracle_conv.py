"""Pins for the oracle's convolution and pooling: brute-force loops, reduction of a 1x1
convolution to a dense layer, the backward pass as the adjoint of the (brute-force pinned) forward pass for every
kernel size and stride in use, finite differences through a conv/pool/conv stage and through a 7x7 stride-2 stem
with global average pooling, pooling ties."""
import numpy as np
import pytest

from oracle import layers as L
from oracle.stage import Stage
from synth_inputs.workloads import AvgPool, Conv2d, Dense, MaxPool2


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


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 1, 3), (2, 3, 7), (1, 2, 5), (2, 0, 1)])
def test_conv_backward_is_the_adjoint_of_the_forward_pass(stride, pad, k):
    """The convolution is linear in x and in W, so <dz, conv(u, W)> = <dx, u> for every u and
    <dz, conv(x, V)> = <dW, V> for every V; with the forward pass pinned by brute force these identities fix dx
    and dW element by element (u and V run over random probes and over unit tensors)."""
    rng = np.random.default_rng(20 + k + stride)
    x = rng.standard_normal((2, 8, 6, 3))
    W = rng.standard_normal((4, k, k, 3))
    zero_b = np.zeros(4)
    z = L.conv2d_forward(x, W, zero_b, stride, pad)
    dz = rng.standard_normal(z.shape)
    dW, db, dx = L.conv2d_backward(dz, x, W, stride, pad)
    assert dW.shape == W.shape and dx.shape == x.shape
    assert np.allclose(db, dz.sum(axis=(0, 1, 2)), atol=1e-12)
    for _ in range(3):
        u, V = rng.standard_normal(x.shape), rng.standard_normal(W.shape)
        assert np.isclose(np.sum(dz * L.conv2d_forward(u, W, zero_b, stride, pad)), np.sum(dx * u), atol=1e-10)
        assert np.isclose(np.sum(dz * L.conv2d_forward(x, V, zero_b, stride, pad)), np.sum(dW * V), atol=1e-10)
    for idx in [(0, 0, 0, 0), (1, 7, 5, 2), (0, 3, 2, 1), (1, 4, 0, 0)]:       # corners, edges, interior
        u = np.zeros(x.shape)
        u[idx] = 1.0
        assert np.isclose(np.sum(dz * L.conv2d_forward(u, W, zero_b, stride, pad)), dx[idx], atol=1e-11)
    for idx in [(0, 0, 0, 0), (3, k - 1, k - 1, 2), (1, k // 2, k // 2, 1), (2, 0, k - 1, 0)]:
        V = np.zeros(W.shape)
        V[idx] = 1.0
        assert np.isclose(np.sum(dz * L.conv2d_forward(x, V, zero_b, stride, pad)), dW[idx], atol=1e-11)


def test_global_average_pooling_values_and_adjoint():
    x = np.zeros((1, 2, 2, 2))
    x[0, :, :, 0] = [[1, 2], [3, 6]]
    x[0, :, :, 1] = [[-1, -1], [-1, 7]]
    assert L.avgpool_forward(x).tolist() == [[3.0, 1.0]]
    dx = L.avgpool_backward(np.array([[4.0, -8.0]]), x.shape)
    assert dx[0, :, :, 0].tolist() == [[1, 1], [1, 1]] and dx[0, :, :, 1].tolist() == [[-2, -2], [-2, -2]]
    rng = np.random.default_rng(6)
    x = rng.standard_normal((3, 4, 5, 2))
    y = L.avgpool_forward(x)
    assert y.shape == (3, 2)
    for n in range(3):
        for c in range(2):
            assert np.isclose(y[n, c], sum(x[n, i, j, c] for i in range(4) for j in range(5)) / 20.0, atol=1e-14)
    dy, u = rng.standard_normal(y.shape), rng.standard_normal(x.shape)
    assert np.isclose(np.sum(dy * L.avgpool_forward(u)), np.sum(L.avgpool_backward(dy, x.shape) * u), atol=1e-12)
    # the [positions, channels] view of the same memory gives the same result
    assert np.array_equal(L.avgpool_forward(x.reshape(3, 20, 2)), y)


def test_stem_and_classifier_head_gradients_match_finite_differences():
    """7x7 stride-2 convolution, pooling, then global average pooling into a dense layer: the layers a
    ResNet-style net has around its bottleneck groups."""
    specs = (Conv2d(2, 3, 8, 8, "gelu", k=7, stride=2, pad=3), MaxPool2(3, 4, 4), AvgPool(3, 4), Dense(3, 2, "none"))
    rng = np.random.default_rng(7)
    params = [rng.standard_normal((3, 7, 7, 2)) * 0.2, rng.standard_normal(3) * 0.1,
              rng.standard_normal((2, 3)) * 0.5, rng.standard_normal(2) * 0.1]
    x = rng.standard_normal((4, 8, 8, 2))
    target = rng.standard_normal((4, 2))

    def loss_of(plist, xin):
        st = Stage(specs, plist, policy="eq1", lam=0.1, lr=0.0, momentum=0.0, n=2)
        out = np.concatenate([st.forward(0, ub, xin[ub * 2:(ub + 1) * 2]) for ub in range(2)])
        return 0.5 * np.sum((out - target) ** 2), out, st

    loss, out, st = loss_of(params, x)
    dx = st.backward(0, out - target)
    h = 1e-6
    for pi, p in enumerate(params):
        for idx in list(np.ndindex(p.shape))[::7]:
            hi = [q.copy() for q in params]
            lo = [q.copy() for q in params]
            hi[pi][idx] += h
            lo[pi][idx] -= h
            fd = (loss_of(hi, x)[0] - loss_of(lo, x)[0]) / (2 * h)
            assert abs(st.g[pi][idx] - fd) < 1e-6, (pi, idx)
    for idx in list(np.ndindex(x.shape))[::11]:
        hi, lo = x.copy(), x.copy()
        hi[idx] += h
        lo[idx] -= h
        fd = (loss_of(params, hi)[0] - loss_of(params, lo)[0]) / (2 * h)
        assert abs(dx[idx] - fd) < 1e-6


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
