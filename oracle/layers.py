"""Textbook layer mathematics in fp64.

The paper gives no formulas for the layers of a stage (Section "Methodology"
only says the layers of a stage run in order, the loss is taken at the last
node and the backward pass runs in reverse), so these are the standard
definitions written out.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

_SQRT2 = np.sqrt(2.0)
_INV_SQRT_2PI = 1.0 / np.sqrt(2.0 * np.pi)


def dense_forward(x, W, b):
    """z[i, o] = sum_k x[i, k] * W[o, k] + b[o]."""
    return x @ W.T + b


def act_forward(z, act):
    if act == "relu":
        return np.maximum(z, 0.0)
    if act == "gelu":
        return 0.5 * z * (1.0 + erf(z / _SQRT2))          # exact (erf) form
    if act == "none":
        return z
    raise ValueError(act)


def act_derivative(z, act):
    if act == "relu":
        return (z > 0.0).astype(np.float64)                # derivative 0 at z = 0
    if act == "gelu":
        return 0.5 * (1.0 + erf(z / _SQRT2)) + z * _INV_SQRT_2PI * np.exp(-0.5 * z * z)
    if act == "none":
        return np.ones_like(z)
    raise ValueError(act)


def dense_backward(dz, x, W_b):
    """Gradients of a dense layer given dz = dL/dz.

    dW[o, k] = sum_i dz[i, o] * x[i, k]   (x: the input saved in forward)
    db[o]    = sum_i dz[i, o]
    dx[i, k] = sum_o dz[i, o] * W_b[o, k] (W_b: the weights the method
                                           prescribes for the backward pass)
    i runs over every leading index (samples, and token positions if there are any).
    """
    dz2, x2 = dz.reshape(-1, dz.shape[-1]), x.reshape(-1, x.shape[-1])
    return dz2.T @ x2, dz2.sum(axis=0), dz @ W_b


def softmax_cross_entropy(logits, labels, denom):
    """Sum over rows of -log softmax(logits)[label], divided by `denom`.

    Returns (loss, dlogits) with dlogits = (softmax - onehot) / denom.  The
    caller passes denom = n * mb so that the loss is the mean over the whole
    mini-batch even when it is evaluated one micro-batch at a time.
    """
    shifted = logits - logits.max(axis=1, keepdims=True)
    logsum = np.log(np.exp(shifted).sum(axis=1, keepdims=True))
    logp = shifted - logsum
    rows = np.arange(logits.shape[0])
    loss = -logp[rows, labels].sum() / denom
    d = np.exp(logp)
    d[rows, labels] -= 1.0
    return loss, d / denom


# ---------------------------------------------------------------------------
# convolution and pooling (NHWC activations, weights [Cout][kh][kw][Cin])
# ---------------------------------------------------------------------------

def conv2d_forward(x, W, b, stride=1, pad=1):
    """Cross-correlation with zero padding, written as the sum over the kernel offsets:
    z[n, oh, ow, o] = b[o] + sum_{i,j,c} x[n, oh*stride + i - pad, ow*stride + j - pad, c] * W[o, i, j, c]."""
    B, H, Wd, _ = x.shape
    Cout, kh, kw, _ = W.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (Wd + 2 * pad - kw) // stride + 1
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    z = np.zeros((B, Ho, Wo, Cout), dtype=np.float64)
    for i in range(kh):
        for j in range(kw):
            patch = xp[:, i:i + stride * Ho:stride, j:j + stride * Wo:stride, :]
            z += patch @ W[:, i, j, :].T
    return z + b


def conv2d_backward(dz, x, W_b, stride=1, pad=1):
    """Gradients of conv2d_forward given dz = dL/dz: (dW, db, dx).

    dW[o,i,j,c] = sum_{n,oh,ow} dz[n,oh,ow,o] * x[n, oh*stride+i-pad, ow*stride+j-pad, c]
    db[o]       = sum_{n,oh,ow} dz[n,oh,ow,o]
    dx          = the same sum scattered back through W_b (the weights the method prescribes)."""
    B, H, Wd, Cin = x.shape
    Cout, kh, kw, _ = W_b.shape
    _, Ho, Wo, _ = dz.shape
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    dxp = np.zeros_like(xp)
    dW = np.zeros((Cout, kh, kw, Cin), dtype=np.float64)
    dz2 = dz.reshape(-1, Cout)
    for i in range(kh):
        for j in range(kw):
            patch = xp[:, i:i + stride * Ho:stride, j:j + stride * Wo:stride, :]
            dW[:, i, j, :] = dz2.T @ patch.reshape(-1, Cin)
            dxp[:, i:i + stride * Ho:stride, j:j + stride * Wo:stride, :] += dz @ W_b[:, i, j, :]
    dx = dxp[:, pad:pad + H, pad:pad + Wd, :]
    return dW, dz2.sum(axis=0), dx


def maxpool2_forward(x):
    """2x2 max pooling, stride 2.  Returns (y, idx) with idx the position of the FIRST maximum in
    the window in row-major order (0: top-left, 1: top-right, 2: bottom-left, 3: bottom-right)."""
    B, H, Wd, C = x.shape
    win = x.reshape(B, H // 2, 2, Wd // 2, 2, C).transpose(0, 1, 3, 2, 4, 5).reshape(B, H // 2, Wd // 2, 4, C)
    idx = np.argmax(win, axis=3)
    y = np.take_along_axis(win, idx[:, :, :, None, :], axis=3)[:, :, :, 0, :]
    return y, idx


def maxpool2_backward(dy, idx, in_shape):
    """Each output gradient goes to the input position that produced the maximum."""
    B, H, Wd, C = in_shape
    dwin = np.zeros((B, H // 2, Wd // 2, 4, C), dtype=np.float64)
    np.put_along_axis(dwin, idx[:, :, :, None, :], dy[:, :, :, None, :], axis=3)
    return dwin.reshape(B, H // 2, Wd // 2, 2, 2, C).transpose(0, 1, 3, 2, 4, 5).reshape(B, H, Wd, C)


def avgpool_forward(x):
    """Global average pooling of an NHWC image (or a [positions, channels] sample): y[n, c] = mean over all
    positions of x[n, ..., c]."""
    B, C = x.shape[0], x.shape[-1]
    return x.reshape(B, -1, C).mean(axis=1)


def avgpool_backward(dy, in_shape):
    """Every position of a sample gets the output gradient of its channel divided by the number of positions."""
    B, C = in_shape[0], in_shape[-1]
    positions = int(np.prod(in_shape[1:-1]))
    dx = np.broadcast_to(dy.reshape(B, 1, C) / positions, (B, positions, C))
    return dx.reshape(in_shape).copy()


def subsample2_forward(x):
    """y[n, i, j, :] = x[n, 2i, 2j, :]: the pixels a stride-2 1x1 convolution reads."""
    return x[:, ::2, ::2, :]


def subsample2_backward(dy, in_shape):
    """The gradient goes back to the pixels that were kept; the others get zero."""
    dx = np.zeros(in_shape, dtype=np.float64)
    dx[:, ::2, ::2, :] = dy
    return dx


# ---------------------------------------------------------------------------
# Layers of the transformer-shaped workload (layer normalisation, causal
# multi-head self-attention); standard definitions, the paper prescribes none.
# ---------------------------------------------------------------------------

LN_EPS = 1e-5


def layernorm_forward(x, gamma, beta, eps=LN_EPS):
    """y[..., d] = gamma[d] * (x[..., d] - mean) / sqrt(var + eps) + beta[d], mean/var over the last axis.
    Returns y and what the backward pass needs: the normalised values and 1/sqrt(var + eps)."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    return xhat * gamma + beta, xhat, rstd


def layernorm_backward(dy, xhat, rstd, gamma_b):
    """Gradients of layernorm_forward; gamma_b is the scale the backward pass is told to use."""
    D = dy.shape[-1]
    dgamma = (dy * xhat).reshape(-1, D).sum(axis=0)
    dbeta = dy.reshape(-1, D).sum(axis=0)
    dxhat = dy * gamma_b
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True) - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dgamma, dbeta, dx


def _split_heads(qkv, heads):
    B, S, D3 = qkv.shape
    D = D3 // 3
    dh = D // heads
    q, k, v = (qkv[:, :, i * D:(i + 1) * D].reshape(B, S, heads, dh).transpose(0, 2, 1, 3) for i in range(3))
    return q, k, v, dh


def attention_probabilities(qkv, heads):
    """softmax over keys j <= i of q_i . k_j / sqrt(head dim), per sequence and head: [B, heads, S, S]."""
    q, k, _, dh = _split_heads(qkv, heads)
    S = qkv.shape[1]
    s = q @ k.transpose(0, 1, 3, 2) / np.sqrt(dh)
    s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def attention_forward(qkv, heads):
    """Causal multi-head self-attention.  qkv: [B, S, 3*D] = (queries | keys | values), each D = heads * dh
    wide with head h in columns h*dh .. (h+1)*dh - 1.  Returns [B, S, D]."""
    B, S, D3 = qkv.shape
    _, _, v, _ = _split_heads(qkv, heads)
    p = attention_probabilities(qkv, heads)
    return (p @ v).transpose(0, 2, 1, 3).reshape(B, S, D3 // 3)


def attention_backward(dout, qkv, heads):
    """Gradient of attention_forward with respect to qkv."""
    B, S, D3 = qkv.shape
    D = D3 // 3
    q, k, v, dh = _split_heads(qkv, heads)
    p = attention_probabilities(qkv, heads)
    do = dout.reshape(B, S, heads, dh).transpose(0, 2, 1, 3)
    dv = p.transpose(0, 1, 3, 2) @ do
    dp = do @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = ds @ k / np.sqrt(dh)
    dk = ds.transpose(0, 1, 3, 2) @ q / np.sqrt(dh)
    back = lambda t: t.transpose(0, 2, 1, 3).reshape(B, S, D)
    return np.concatenate([back(dq), back(dk), back(dv)], axis=-1)


# ---------------------------------------------------------------------------
# Batch normalisation (training mode) for the bottleneck-shaped workload: statistics over all rows
# (samples x positions) of what one forward call sees, per channel.  Standard definition.
# ---------------------------------------------------------------------------

BN_EPS = 1e-5


def batchnorm_forward(x, gamma, beta, eps=BN_EPS):
    """x: [..., C]; y = gamma * (x - mean_c) / sqrt(var_c + eps) + beta with mean/var over every leading index
    (biased variance).  Returns y, the normalised values and 1/sqrt(var + eps) per channel."""
    C = x.shape[-1]
    x2 = x.reshape(-1, C)
    mu = x2.mean(axis=0)
    var = ((x2 - mu) ** 2).mean(axis=0)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, xhat, rstd


def batchnorm_backward(dy, xhat, rstd, gamma_b):
    """Gradients of batchnorm_forward; gamma_b is the scale the backward pass is told to use."""
    C = dy.shape[-1]
    dy2, xh2 = dy.reshape(-1, C), xhat.reshape(-1, C)
    R = dy2.shape[0]
    dgamma = (dy2 * xh2).sum(axis=0)
    dbeta = dy2.sum(axis=0)
    dx = (gamma_b * rstd / R) * (R * dy - dbeta - xhat * dgamma)
    return dgamma, dbeta, dx
