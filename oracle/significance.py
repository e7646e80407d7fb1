"""Significance of stale weights and the intermediate-weight coefficients.

Section "I-TiMePReSt", Eq. 2 and Appendix A.1: the significance of weights
that are stale by degree delta >= 0 decays at a rate proportional to its
current value, f(0) = 1, which in the limit of many small steps gives
f(delta) = exp(-lambda * delta) with lambda > 0; f lies in (0, 1].

Section "I-TiMePReSt", Eq. 1 and Appendix A.2: the intermediate weight used by
the backward pass is (2 - 1/f(delta)) times the stale weight.

The degree of staleness is taken as the number of updates applied to the
stage between the version the forward pass used and the latest version when
the backward pass runs (the paper's example W_2(1|3): forward on the update
of mini-batch 1, latest is the update of mini-batch 3, delta = 2).
"""
from __future__ import annotations

import math

POLICIES = ("latest", "eq1", "convex", "stashed")   # the policies that fix the backward weights from (v_f, latest, delta)


def f(delta: float, lam: float) -> float:
    """Eq. 2: significance of weights stale by `delta`."""
    if delta < 0 or lam <= 0:
        raise ValueError("delta >= 0 and lambda > 0 required")
    return math.exp(-lam * delta)


def f_finite(delta: float, lam: float, n: int) -> float:
    """Appendix A.1 before the limit: (1 - lambda*delta/n)^n, n steps of size delta/n."""
    return (1.0 - lam * delta / n) ** n


def coefficients(policy: str, delta: int, lam: float):
    """(alpha, beta) of W_b = alpha * W_stale + beta * W_latest.

    latest   V-TiMePReSt: the backward pass runs on the latest weights.
    eq1      I-TiMePReSt as printed (Eq. 1): W_b = (2 - 1/f) * W_stale.
    convex   I-TiMePReSt read as the blend the prose describes (Appendix A.2:
             the stale weight scaled by its significance f, the remaining
             share 1 - f given to the latest weights).
    stashed  backward on the very weights the forward used (PipeDream-style
             horizontal stashing, the scheme the paper compares against).
    """
    if policy == "latest":
        return 0.0, 1.0
    if policy == "stashed":
        return 1.0, 0.0
    fd = f(delta, lam)
    if policy == "eq1":
        return 2.0 - 1.0 / fd, 0.0
    if policy == "convex":
        return fd, 1.0 - fd
    raise ValueError(f"unknown policy {policy!r}")
