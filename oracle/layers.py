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
    """
    return dz.T @ x, dz.sum(axis=0), dz @ W_b


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
