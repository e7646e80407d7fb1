"""Pins of the oracle's batch normalisation and of the identity-bottleneck block built from it (1x1
convolutions as per-position dense layers, 3x3 convolution, residual add followed by ReLU): index
loops, invariances, finite differences."""
import math

import numpy as np

from oracle import layers as L
from oracle.stage import Stage
from synth_inputs import workloads as W

RNG = np.random.default_rng(21)


def test_batchnorm_forward_brute_force_and_invariances():
    x = RNG.standard_normal((3, 5, 4)) * 1.5 + 0.7
    gamma, beta = RNG.standard_normal(4), RNG.standard_normal(4)
    y, xhat, rstd = L.batchnorm_forward(x, gamma, beta)
    for c in range(4):
        vals = [x[b, t, c] for b in range(3) for t in range(5)]
        mu = sum(vals) / 15
        var = sum((v - mu) ** 2 for v in vals) / 15
        assert abs(rstd[c] - 1 / math.sqrt(var + 1e-5)) < 1e-12
        for b in range(3):
            for t in range(5):
                assert abs(y[b, t, c] - (gamma[c] * (x[b, t, c] - mu) / math.sqrt(var + 1e-5) + beta[c])) < 1e-12
    assert np.allclose(xhat.reshape(-1, 4).mean(0), 0, atol=1e-12)
    # per-channel shift of the input changes nothing; the statistics couple the samples: changing one
    # sample changes the output of the others
    y2, _, _ = L.batchnorm_forward(x + np.array([1.0, -2.0, 3.0, 0.5]), gamma, beta)
    assert np.allclose(y, y2, atol=1e-10)
    x3 = x.copy(); x3[0] += 1.0
    assert not np.allclose(L.batchnorm_forward(x3, gamma, beta)[0][1:], y[1:])
    # same numbers whether a sample is [positions, channels] or an [h, w, channels] image
    y4, _, _ = L.batchnorm_forward(x.reshape(3, 5, 1, 4), gamma, beta)
    assert np.array_equal(y4.reshape(y.shape), y)


def test_batchnorm_backward_finite_differences():
    x = RNG.standard_normal((2, 3, 5))
    gamma, beta = RNG.standard_normal(5) + 1.0, RNG.standard_normal(5)
    c = RNG.standard_normal((2, 3, 5))
    f = lambda xx, gg, bb: float((L.batchnorm_forward(xx, gg, bb)[0] * c).sum())
    _, xhat, rstd = L.batchnorm_forward(x, gamma, beta)
    dgamma, dbeta, dx = L.batchnorm_backward(c, xhat, rstd, gamma)
    h = 1e-6
    for idx in [(0, 0, 0), (1, 2, 4), (0, 1, 2), (1, 0, 3)]:
        e = np.zeros_like(x); e[idx] = h
        assert abs((f(x + e, gamma, beta) - f(x - e, gamma, beta)) / (2 * h) - dx[idx]) < 1e-6
    for d in range(5):
        e = np.zeros(5); e[d] = h
        assert abs((f(x, gamma + e, beta) - f(x, gamma - e, beta)) / (2 * h) - dgamma[d]) < 1e-6
        assert abs((f(x, gamma, beta + e) - f(x, gamma, beta - e)) / (2 * h) - dbeta[d]) < 1e-6
    assert np.allclose(dx.reshape(-1, 5).sum(0), 0, atol=1e-12)         # a channel shift does not move the output
    _, _, dx2 = L.batchnorm_backward(c, xhat, rstd, 3.0 * gamma)
    assert np.allclose(dx2, 3.0 * dx)                                    # linear in the backward scale


def _block(seed=5):
    blk = W.bottleneck_block(8, 4, 2, 2)
    w = W.Workload(name="bneck_pin", dtype="f32", stages=(blk,), mb=3, n=2, classes=2)
    rng = np.random.default_rng(seed)
    params = [p + 0.2 * rng.standard_normal(p.shape) for p in W.init_params(w, 0)]
    return blk, params


def test_bottleneck_block_gradients_finite_differences():
    blk, params = _block()
    x = np.random.default_rng(6).standard_normal((6, 4, 8)) + 0.3
    c = np.random.default_rng(7).standard_normal((6, 4, 8))

    def loss(ps, xx):
        st = Stage(blk, ps, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=2)
        ys = [st.forward(0, ub, xx[ub * 3:(ub + 1) * 3]) for ub in range(2)]
        return float((np.concatenate(ys).reshape(c.shape) * c).sum())

    st = Stage(blk, params, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=2)
    for ub in range(2):
        st.forward(0, ub, x[ub * 3:(ub + 1) * 3])
    dx = st.backward(0, c).reshape(x.shape)
    h = 1e-6
    for pi in range(len(params)):
        for fi in (0, params[pi].size // 2, params[pi].size - 1):
            idx = np.unravel_index(fi, params[pi].shape)
            hi = [p.copy() for p in params]; lo = [p.copy() for p in params]
            hi[pi][idx] += h; lo[pi][idx] -= h
            num = (loss(hi, x) - loss(lo, x)) / (2 * h)
            assert abs(num - st.g[pi][idx]) < 5e-6 * max(1.0, abs(num)), (pi, idx, num, st.g[pi][idx])
    for idx in [(0, 0, 0), (5, 3, 7), (2, 1, 4), (3, 2, 1)]:
        e = np.zeros_like(x); e[idx] = h
        num = (loss(params, x + e) - loss(params, x - e)) / (2 * h)
        assert abs(num - dx[idx]) < 5e-6 * max(1.0, abs(num))


def test_micro_batches_are_normalised_separately():
    # the statistics belong to one forward call: the first micro-batch's output does not depend on the second
    blk, params = _block()
    x = np.random.default_rng(8).standard_normal((6, 4, 8))
    st = Stage(blk, params, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=2)
    y0 = st.forward(0, 0, x[:3])
    st2 = Stage(blk, params, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=2)
    x2 = x.copy(); x2[3:] += 5.0
    assert np.array_equal(st2.forward(0, 0, x2[:3]), y0)


def test_block_with_zero_branch_is_relu_of_input():
    blk, params = _block()
    params = [p.copy() for p in params]
    params[10][...] = 0.0; params[11][...] = 0.0            # last batch norm: scale and shift zero
    st = Stage(blk, params, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=1)
    x = np.random.default_rng(9).standard_normal((3, 4, 8))
    assert np.array_equal(st.forward(0, 0, x).reshape(x.shape), np.maximum(x, 0.0))


# ---- first block of a group: stride 2 on the 3x3, projection shortcut ---------------------------------------

def test_subsample_brute_force_adjoint_and_strided_1x1_convolution():
    x = RNG.standard_normal((2, 4, 6, 3))
    y = L.subsample2_forward(x)
    assert y.shape == (2, 2, 3, 3)
    for n in range(2):
        for i in range(2):
            for j in range(3):
                assert np.array_equal(y[n, i, j], x[n, 2 * i, 2 * j])
    # a 1x1 convolution with stride 2, no padding and the identity as weights reads exactly these pixels
    assert np.array_equal(L.conv2d_forward(x, np.eye(3).reshape(3, 1, 1, 3), np.zeros(3), stride=2, pad=0), y)
    # backward is the adjoint: <sub(x), dy> = <x, sub^T(dy)>, and nothing lands on the dropped pixels
    dy = RNG.standard_normal(y.shape)
    dx = L.subsample2_backward(dy, x.shape)
    assert abs((y * dy).sum() - (x * dx).sum()) < 1e-12
    assert np.count_nonzero(dx[:, 1::2]) == 0 and np.count_nonzero(dx[:, :, 1::2]) == 0


def _down_block(seed=15):
    blk = W.bottleneck_down_block(4, 4, 8, 4, 4)
    w = W.Workload(name="bneck_down_pin", dtype="f32", stages=(blk,), mb=3, n=2, classes=2)
    rng = np.random.default_rng(seed)
    params = [p + 0.2 * rng.standard_normal(p.shape) for p in W.init_params(w, 0)]
    return blk, params


def test_down_block_gradients_finite_differences():
    blk, params = _down_block()
    assert [l.kind for l in blk] == ["res", "dense", "bn", "conv", "bn", "dense", "bn", "swap", "sub", "dense", "bn", "res"]
    x = np.random.default_rng(16).standard_normal((6, 16, 4)) + 0.3
    c = np.random.default_rng(17).standard_normal((6, 4, 8))

    def loss(ps, xx):
        st = Stage(blk, ps, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=2)
        ys = [st.forward(0, ub, xx[ub * 3:(ub + 1) * 3]) for ub in range(2)]
        return float((np.concatenate(ys).reshape(c.shape) * c).sum())

    st = Stage(blk, params, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=2)
    for ub in range(2):
        assert st.forward(0, ub, x[ub * 3:(ub + 1) * 3]).size == 3 * 4 * 8
    dx = st.backward(0, c).reshape(x.shape)
    h = 1e-6
    for pi in range(len(params)):
        for fi in (0, params[pi].size // 2, params[pi].size - 1):
            idx = np.unravel_index(fi, params[pi].shape)
            hi = [p.copy() for p in params]; lo = [p.copy() for p in params]
            hi[pi][idx] += h; lo[pi][idx] -= h
            num = (loss(hi, x) - loss(lo, x)) / (2 * h)
            assert abs(num - st.g[pi][idx]) < 5e-6 * max(1.0, abs(num)), (pi, idx, num, st.g[pi][idx])
    # every input pixel: the odd ones reach the output through the 3x3 only, the even ones through both branches
    for idx in [(0, 0, 0), (5, 15, 3), (2, 5, 1), (3, 10, 2), (1, 3, 0), (4, 8, 3)]:
        e = np.zeros_like(x); e[idx] = h
        num = (loss(params, x + e) - loss(params, x - e)) / (2 * h)
        assert abs(num - dx[idx]) < 5e-6 * max(1.0, abs(num)), (idx, num, dx[idx])


def test_down_block_branches_separately():
    blk, params = _down_block()
    x = np.random.default_rng(18).standard_normal((3, 16, 4))
    # main branch switched off (last batch norm of the main branch: scale and shift zero): what is left is the
    # shortcut -- subsample, 1x1 projection, batch norm -- written out here without the stage
    p = [q.copy() for q in params]
    p[10][...] = 0.0; p[11][...] = 0.0
    st = Stage(blk, p, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=1)
    y = st.forward(0, 0, x).reshape(3, 2, 2, 8)
    xs = x.reshape(3, 4, 4, 4)[:, ::2, ::2, :]
    z = xs @ p[12].T + p[13]
    zz = z.reshape(-1, 8)
    bn = (z - zz.mean(0)) / np.sqrt(zz.var(0) + 1e-5) * p[14] + p[15]
    assert np.allclose(y, np.maximum(bn, 0.0), atol=1e-12)
    # shortcut switched off: the output no longer depends on the projection weights, and it does depend on odd pixels
    p = [q.copy() for q in params]
    p[14][...] = 0.0; p[15][...] = 0.0
    y1 = Stage(blk, p, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=1).forward(0, 0, x)
    p2 = [q.copy() for q in p]; p2[12] += 1.0
    assert np.array_equal(Stage(blk, p2, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=1).forward(0, 0, x), y1)
    x2 = x.copy(); x2[:, 5, :] += 1.0                       # pixel (1, 1): dropped by the shortcut, seen by the 3x3
    assert not np.allclose(Stage(blk, p, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=1).forward(0, 0, x2), y1)
