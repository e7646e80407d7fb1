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
