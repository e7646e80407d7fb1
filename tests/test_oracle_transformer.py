"""Pins of the oracle's transformer layers (layer normalisation, causal multi-head attention, residual
connections, per-token dense layers) against things other than themselves: brute-force loops over
indices, invariances the definitions imply, and central finite differences of a scalar loss through
whole blocks.  A dropped term, a wrong sign, a transposed operand or a leaking causal mask fails one."""
import math

import numpy as np
import pytest

from oracle import layers as L
from oracle.stage import Stage
from synth_inputs import workloads as W

RNG = np.random.default_rng(11)


def test_layernorm_forward_brute_force_and_invariances():
    x = RNG.standard_normal((3, 4, 7)) * 2.0 + 0.5
    gamma, beta = RNG.standard_normal(7), RNG.standard_normal(7)
    y, xhat, rstd = L.layernorm_forward(x, gamma, beta)
    for b in range(3):
        for t in range(4):
            row = x[b, t]
            mu = sum(row) / 7
            var = sum((v - mu) ** 2 for v in row) / 7
            for d in range(7):
                assert abs(y[b, t, d] - (gamma[d] * (row[d] - mu) / math.sqrt(var + 1e-5) + beta[d])) < 1e-12
    # normalised values: zero mean, variance var/(var+eps); shifting a row changes nothing, scaling it
    # changes nothing but for eps
    assert np.allclose(xhat.mean(-1), 0, atol=1e-12)
    y2, _, _ = L.layernorm_forward(x + 3.7, gamma, beta)
    assert np.allclose(y, y2, atol=1e-10)
    y3, _, _ = L.layernorm_forward(x * 5.0, gamma, beta, eps=0.0)
    y0, _, _ = L.layernorm_forward(x, gamma, beta, eps=0.0)
    assert np.allclose(y3, y0, atol=1e-10)


def test_layernorm_backward_finite_differences_and_orthogonality():
    x = RNG.standard_normal((2, 3, 6))
    gamma, beta = RNG.standard_normal(6) + 1.0, RNG.standard_normal(6)
    c = RNG.standard_normal((2, 3, 6))
    f = lambda xx, gg, bb: float((L.layernorm_forward(xx, gg, bb)[0] * c).sum())
    _, xhat, rstd = L.layernorm_forward(x, gamma, beta)
    dgamma, dbeta, dx = L.layernorm_backward(c, xhat, rstd, gamma)
    h = 1e-6
    for idx in [(0, 0, 0), (1, 2, 5), (0, 1, 3)]:
        e = np.zeros_like(x); e[idx] = h
        assert abs((f(x + e, gamma, beta) - f(x - e, gamma, beta)) / (2 * h) - dx[idx]) < 1e-6
    for d in range(6):
        e = np.zeros(6); e[d] = h
        assert abs((f(x, gamma + e, beta) - f(x, gamma - e, beta)) / (2 * h) - dgamma[d]) < 1e-6
        assert abs((f(x, gamma, beta + e) - f(x, gamma, beta - e)) / (2 * h) - dbeta[d]) < 1e-6
    # the output does not move when a row is shifted: dx sums to zero along the features
    assert np.allclose(dx.sum(-1), 0, atol=1e-12)


def _attention_loops(qkv, heads):
    B, S, D3 = qkv.shape
    D = D3 // 3
    dh = D // heads
    out = np.zeros((B, S, D))
    for b in range(B):
        for h in range(heads):
            for i in range(S):
                q = qkv[b, i, h * dh:(h + 1) * dh]
                scores = [sum(q[d] * qkv[b, j, D + h * dh + d] for d in range(dh)) / math.sqrt(dh) for j in range(i + 1)]
                m = max(scores)
                e = [math.exp(s - m) for s in scores]
                z = sum(e)
                for d in range(dh):
                    out[b, i, h * dh + d] = sum(e[j] / z * qkv[b, j, 2 * D + h * dh + d] for j in range(i + 1))
    return out


def test_attention_forward_brute_force_causality_and_rows():
    qkv = RNG.standard_normal((2, 5, 3 * 8))
    out = L.attention_forward(qkv, 2)
    assert np.allclose(out, _attention_loops(qkv, 2), atol=1e-12)
    p = L.attention_probabilities(qkv, 2)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-12)
    assert np.all(p[:, :, np.triu_indices(5, 1)[0], np.triu_indices(5, 1)[1]] == 0.0)
    # the first token attends only to itself: its output is its own value vector
    assert np.allclose(out[:, 0, :], qkv[:, 0, 16:], atol=1e-12)
    # changing a later token leaves earlier outputs alone
    q2 = qkv.copy(); q2[:, 3:, :] += 1.0
    assert np.array_equal(L.attention_forward(q2, 2)[:, :3], out[:, :3])
    # heads do not mix: permuting heads in the input permutes them in the output
    perm = np.concatenate([np.arange(4, 8), np.arange(0, 4)])
    q3 = np.concatenate([qkv[..., 0:8][..., perm], qkv[..., 8:16][..., perm], qkv[..., 16:24][..., perm]], axis=-1)
    assert np.allclose(L.attention_forward(q3, 2), out[..., perm], atol=1e-12)


def test_attention_backward_finite_differences():
    qkv = RNG.standard_normal((2, 4, 3 * 6))
    c = RNG.standard_normal((2, 4, 6))
    f = lambda t: float((L.attention_forward(t, 3) * c).sum())
    g = L.attention_backward(c, qkv, 3)
    h = 1e-6
    for idx in [(0, 0, 0), (1, 3, 5), (0, 2, 7), (1, 1, 11), (0, 3, 13), (1, 0, 17), (0, 1, 9)]:
        e = np.zeros_like(qkv); e[idx] = h
        assert abs((f(qkv + e) - f(qkv - e)) / (2 * h) - g[idx]) < 1e-6, idx


def _block_stage(policy="latest"):
    blk = W.transformer_block(8, 2, 12, 3)
    w = W.Workload(name="tfm_pin", dtype="f32", stages=(blk,), mb=2, n=2, classes=2)
    params = W.init_params(w, 0)
    rng = np.random.default_rng(5)
    params = [p + 0.1 * rng.standard_normal(p.shape) for p in params]     # biases, scale and shift away from 0 / 1
    return blk, params


def test_block_gradients_finite_differences():
    blk, params = _block_stage()
    x = np.random.default_rng(6).standard_normal((4, 3, 8))
    c = np.random.default_rng(7).standard_normal((4, 3, 8))

    def loss(ps, xx):
        st = Stage(blk, ps, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=2)
        ys = [st.forward(0, ub, xx[ub * 2:(ub + 1) * 2]) for ub in range(2)]
        return float((np.concatenate(ys) * c).sum())

    st = Stage(blk, params, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=2)
    for ub in range(2):
        st.forward(0, ub, x[ub * 2:(ub + 1) * 2])
    dx = st.backward(0, c)
    h = 1e-6
    for pi in range(len(params)):
        flat_idx = [0, params[pi].size // 2, params[pi].size - 1]
        for fi in flat_idx:
            idx = np.unravel_index(fi, params[pi].shape)
            hi = [p.copy() for p in params]; lo = [p.copy() for p in params]
            hi[pi][idx] += h; lo[pi][idx] -= h
            num = (loss(hi, x) - loss(lo, x)) / (2 * h)
            assert abs(num - st.g[pi][idx]) < 2e-6 * max(1.0, abs(num)), (pi, idx, num, st.g[pi][idx])
    for idx in [(0, 0, 0), (3, 2, 7), (1, 1, 4)]:
        e = np.zeros_like(x); e[idx] = h
        num = (loss(params, x + e) - loss(params, x - e)) / (2 * h)
        assert abs(num - dx[idx]) < 2e-6 * max(1.0, abs(num))


def test_residual_is_identity_plus_branch():
    # a block whose branch outputs are zero (projection and second FFN weights and biases zero) is the identity
    blk, params = _block_stage()
    params = [p.copy() for p in params]
    shapes = [p.shape for p in params]
    # parameter order: ln1 (g, b), qkv (W, b), proj (W, b), ln2 (g, b), ffn1 (W, b), ffn2 (W, b)
    for i in (4, 5, 10, 11):
        params[i][...] = 0.0
    st = Stage(blk, params, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=1)
    x = np.random.default_rng(8).standard_normal((2, 3, 8))
    assert np.array_equal(st.forward(0, 0, x), x)
    dx = st.backward(0, np.ones_like(x))
    assert np.array_equal(dx, np.ones_like(x))          # only the skip path carries gradient
    assert shapes[2] == (24, 8) and shapes[8] == (12, 8)


def test_per_token_dense_equals_dense_on_flattened_rows():
    x = RNG.standard_normal((3, 4, 5))
    Wm, b = RNG.standard_normal((6, 5)), RNG.standard_normal(6)
    z = L.dense_forward(x, Wm, b)
    assert np.allclose(z.reshape(12, 6), L.dense_forward(x.reshape(12, 5), Wm, b), atol=1e-14)
    dz = RNG.standard_normal((3, 4, 6))
    dW, db, dx = L.dense_backward(dz, x, Wm)
    dW2, db2, dx2 = L.dense_backward(dz.reshape(12, 6), x.reshape(12, 5), Wm)
    assert np.allclose(dW, dW2) and np.allclose(db, db2) and np.allclose(dx.reshape(12, 5), dx2)


def test_intermediate_weights_enter_layernorm_backward_through_scale_only():
    # under a stashing policy with staleness, dx of a LayerNorm is linear in the backward scale and the
    # parameter gradients do not depend on it
    ln = (W.LayerNorm(6, 2),)
    g0, b0 = np.ones(6) + 0.1 * RNG.standard_normal(6), 0.1 * RNG.standard_normal(6)
    x = RNG.standard_normal((2, 2, 6)); dy = RNG.standard_normal((2, 2, 6))
    _, xhat, rstd = L.layernorm_forward(x, g0, b0)
    dg1, db1, dx1 = L.layernorm_backward(dy, xhat, rstd, g0)
    dg2, db2, dx2 = L.layernorm_backward(dy, xhat, rstd, 2.0 * g0)
    assert np.array_equal(dg1, dg2) and np.array_equal(db1, db2) and np.allclose(dx2, 2.0 * dx1)
    st = Stage(ln, [g0, b0], policy="convex", lam=0.3, lr=0.1, momentum=0.0, n=1)
    assert st.pidx == [0]
