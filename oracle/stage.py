"""One pipeline stage under the V-TiMePReSt / I-TiMePReSt weight rules (fp64).

Follows, in event order:
  forward   Section "V-TiMePReSt" / "I-TiMePReSt": every micro-batch forward
            reads the latest weights present at the stage; under the
            I-policies that version is kept (stashed) for the mini-batch.
  backward  one pass for the whole mini-batch (Section "Methodology"), on the
            latest weights (V) or on the intermediate weights built from the
            stashed version and the degree of staleness (I; Eq. 1-2).  The
            activations saved in forward are reused as they are; the
            prescribed weights enter through dx = dz . W_b.
  retention Section "Memory Overhead": a stale version stays until the last
            mini-batch that used it in forward has built its intermediate
            weights; V keeps nothing but the latest version.
  update    after every mini-batch (Section "Pipeline Parallelism"): SGD with
            momentum applied to the latest weights, producing the next
            version.  The paper names no optimiser; the form is
            m <- mu*m + g, W <- W - lr*m (m starts at zero).

Parameters of a stage are a flat list [W0, b0, W1, b1, ...]; every entry is
versioned, stashed and blended alike.

Policy "timeprest" is the parent method as Sections "Methodology" and
"V-TiMePReSt" (Challenge 1) describe it: no horizontal stashing (forward and
backward of a mini-batch may read different versions) but a pass cannot pick
up updates that happen while it is under way -- every stage of a pass reads
the version that was the latest THERE when the pass started.  Which version
that is, is known to whoever drives the stages (pipeline.py takes the
snapshot when a pass starts); the stage is told the version per call and
keeps it alive through pin()/unpin().
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

from . import layers as L
from .significance import coefficients


class StageError(RuntimeError):
    pass


class Stage:
    def __init__(self, layer_specs, params: List[np.ndarray], *, policy: str, lam: float,
                 lr: float, momentum: float, n: int, first_stage: bool = False, storage=None):
        """storage: optional rounding (e.g. to bfloat16) applied wherever the workload keeps a tensor
        in its activation type -- weight compute copies, layer outputs, propagated gradients -- while all
        arithmetic stays fp64.  It puts decisions that hinge on stored values (which element of a
        pooling window is the maximum) in the precision the workload prescribes; None keeps pure fp64."""
        self.q = storage if storage is not None else (lambda a: a)
        self.specs = list(layer_specs)
        # position of each layer's weight in the flat parameter list (None: layer has no parameters)
        self.pidx, nxt = [], 0
        for spec in self.specs:
            if getattr(spec, "kind", "dense") in ("pool", "attn", "res", "sub", "swap", "avg"):
                self.pidx.append(None)
            else:
                self.pidx.append(nxt)
                nxt += 2
        self.policy = policy
        self.lam = float(lam)
        self.lr = float(lr)
        self.mu = float(momentum)
        self.n = int(n)
        self.first_stage = first_stage
        self.latest = 0                                    # number of updates applied
        self.weights: Dict[int, List[np.ndarray]] = {0: [np.array(p, dtype=np.float64) for p in params]}
        self.refcnt: Dict[int, int] = {0: 0}               # forward users that have not blended yet
        self.m = [np.zeros_like(p) for p in self.weights[0]]
        self.g: Optional[List[np.ndarray]] = None          # gradient of the last backward
        self.inflight: Dict[int, dict] = {}                # mini-batch -> forward record
        self.evicted: List[int] = []
        self.last_W_b: Optional[List[np.ndarray]] = None
        self.trace: List[tuple] = []                       # (event, mb, v_f, v_now, delta)

    # -- forward ---------------------------------------------------------
    def pin(self, version: int) -> None:
        """One more user of `version` (it stays in memory until unpinned and no longer the latest)."""
        if version not in self.weights:
            raise StageError(f"version {version} is not held")
        self.refcnt[version] += 1

    def unpin(self, version: int) -> None:
        if self.refcnt.get(version, 0) <= 0:
            raise StageError(f"version {version} has no user to drop")
        self.refcnt[version] -= 1
        self._evict_if_unused(version)

    def forward(self, mb: int, ub: int, x: np.ndarray, version: Optional[int] = None) -> np.ndarray:
        """version: the weights to read, for policy "timeprest" (default: the latest at the stage)."""
        if version is not None and self.policy != "timeprest":
            raise StageError("only the timeprest policy names the version of a pass")
        rec = self.inflight.get(mb)
        if rec is None:
            if ub != 0:
                raise StageError("micro-batches of a mini-batch must arrive in order")
            rec = {"v_f": self.latest, "saved": [], "versions": []}
            self.inflight[mb] = rec
            if version is not None:
                rec["v_f"] = version
            if self.policy not in ("latest", "timeprest"):
                self.refcnt[self.latest] += 1              # stash: one user per mini-batch
        if ub != len(rec["saved"]) or ub >= self.n:
            raise StageError("micro-batch index out of order")
        if self.policy not in ("latest", "timeprest") and rec["v_f"] != self.latest:
            raise StageError("update landed between micro-batches of one mini-batch")
        v_read = self.latest if version is None else version
        if v_read not in self.weights:
            raise StageError(f"version {v_read} is not held")
        W = [self.q(p) if p.ndim > 1 else p for p in self.weights[v_read]]        # compute copy
        rec["versions"].append(v_read)
        saved = []
        outs = []                                          # inspection only: every layer's stored output, in layer order
        rec.setdefault("outs", []).append(outs)
        a = np.asarray(x, dtype=np.float64)
        skip = None                                        # activation remembered by a residual "begin"
        for li, spec in enumerate(self.specs):
            kind = getattr(spec, "kind", "dense")
            pi = self.pidx[li]
            if hasattr(spec, "in_shape"):                  # same memory, the layer's own view of a sample
                a = a.reshape((a.shape[0],) + tuple(spec.in_shape()))
            if kind == "pool":
                y, idx = L.maxpool2_forward(a)
                saved.append((a.shape, idx))
                a = y
                outs.append(a)
                continue
            if kind == "sub":
                saved.append((a.shape,))
                a = L.subsample2_forward(a)
                outs.append(a)
                continue
            if kind == "avg":
                saved.append((a.shape,))
                a = self.q(L.avgpool_forward(a))
                outs.append(a)
                continue
            if kind == "swap":                             # projection shortcut: the second branch starts from the
                saved.append(None)                         # remembered tensor, the main branch's result waits for the add
                a, skip = skip, a
                outs.append(a)
                continue
            if kind == "res":
                if spec.mark == "begin":
                    skip = a
                    saved.append(None)
                else:
                    z = a + skip.reshape(a.shape)
                    saved.append((None, z))
                    a = self.q(L.act_forward(z, spec.act))
                outs.append(a)
                continue
            if kind == "bn":
                y, xhat, rstd = L.batchnorm_forward(a, W[pi], W[pi + 1])
                saved.append((xhat, rstd, y))
                a = self.q(L.act_forward(y, spec.act))
                outs.append(a)
                continue
            if kind == "ln":
                y, xhat, rstd = L.layernorm_forward(a, W[pi], W[pi + 1])
                saved.append((xhat, rstd))
                a = self.q(y)
                outs.append(a)
                continue
            if kind == "attn":
                saved.append((a,))
                a = self.q(L.attention_forward(a, spec.heads))
                outs.append(a)
                continue
            if kind == "conv":
                z = L.conv2d_forward(a, W[pi], W[pi + 1], spec.stride, spec.pad)
            else:
                z = L.dense_forward(a, W[pi], W[pi + 1])
            saved.append((a, z))
            a = self.q(L.act_forward(z, spec.act))
            outs.append(a)
        rec["saved"].append(saved)
        return a

    # -- backward weights ------------------------------------------------
    def backward_weights(self, mb: int, version: Optional[int] = None):
        """W_b for mini-batch mb and the (v_f, v_now, delta) triple behind it."""
        rec = self.inflight[mb]
        v_now = self.latest
        if self.policy == "timeprest":                     # the version the backward pass started on, as it is
            v_b = v_now if version is None else version
            if v_b not in self.weights:
                raise StageError(f"version {v_b} is not held")
            return self.weights[v_b], (rec["versions"][0], v_b, 0)
        if self.policy == "latest":
            return self.weights[v_now], (rec["versions"][0], v_now, 0)
        v_f = rec["v_f"]
        if v_f not in self.weights:
            raise StageError(f"version {v_f} is no longer stashed")
        delta = v_now - v_f
        alpha, beta = coefficients(self.policy, delta, self.lam)
        stale, latest = self.weights[v_f], self.weights[v_now]
        if delta == 0:
            W_b = [s.copy() for s in stale]                # no staleness: stale = latest = intermediate
        else:
            W_b = [alpha * s + beta * l for s, l in zip(stale, latest)]
        return W_b, (v_f, v_now, delta)

    # -- backward --------------------------------------------------------
    def backward(self, mb: int, dy: np.ndarray, version: Optional[int] = None) -> Optional[np.ndarray]:
        rec = self.inflight.get(mb)
        if rec is None or len(rec["saved"]) != self.n:
            raise StageError("backward needs all n micro-batch forwards of the mini-batch")
        if version is not None and self.policy != "timeprest":
            raise StageError("only the timeprest policy names the version of a pass")
        W_b, (v_f, v_now, delta) = self.backward_weights(mb, version)
        self.last_W_b = W_b
        W_b = [self.q(p) if p.ndim > 1 else p for p in W_b]                       # compute copy
        self.trace.append(("B", mb, v_f, v_now, delta))
        dy = np.asarray(dy, dtype=np.float64)
        rows = dy.shape[0] // self.n                       # samples per micro-batch
        g = [np.zeros_like(p) for p in self.weights[self.latest]]
        dx_parts = []
        for ub in range(self.n):                           # one backward, all micro-batches
            da = dy[ub * rows:(ub + 1) * rows]
            saved = rec["saved"][ub]
            dskip = None                                   # gradient that flows around a residual branch
            for li in reversed(range(len(self.specs))):
                spec = self.specs[li]
                kind = getattr(spec, "kind", "dense")
                pi = self.pidx[li]
                if hasattr(spec, "out_shape"):
                    da = da.reshape((da.shape[0],) + tuple(spec.out_shape()))
                if dskip is not None:
                    dskip = dskip.reshape(da.shape) if dskip.size == da.size else dskip
                if kind == "pool":
                    in_shape, idx = saved[li]
                    da = L.maxpool2_backward(da, idx, in_shape)
                    continue
                if kind == "sub":
                    da = L.subsample2_backward(da, saved[li][0])
                    continue
                if kind == "avg":
                    da = self.q(L.avgpool_backward(da, saved[li][0]))
                    continue
                if kind == "swap":                         # da: gradient of the remembered tensor through the second
                    da, dskip = dskip, da                  # branch, kept for the begin; the main branch goes on
                    da = da.reshape((da.shape[0],) + tuple(spec.in_shape()))
                    continue
                if kind == "res":
                    if spec.mark == "add":
                        da = self.q(da * L.act_derivative(saved[li][1], spec.act))
                        dskip = da
                    else:
                        da = self.q(da + dskip.reshape(da.shape))
                        dskip = None
                    continue
                if kind == "bn":
                    xhat, rstd, y = saved[li]
                    dyv = self.q(da * L.act_derivative(y, spec.act))
                    dgamma, dbeta, da = L.batchnorm_backward(dyv, xhat, rstd, W_b[pi])
                    g[pi] += dgamma
                    g[pi + 1] += dbeta
                    da = self.q(da)
                    continue
                if kind == "ln":
                    xhat, rstd = saved[li]
                    dgamma, dbeta, da = L.layernorm_backward(da, xhat, rstd, W_b[pi])
                    g[pi] += dgamma
                    g[pi + 1] += dbeta
                    da = self.q(da)
                    continue
                if kind == "attn":
                    da = self.q(L.attention_backward(da, saved[li][0], spec.heads))
                    continue
                x_in, z = saved[li]
                dz = self.q(da * L.act_derivative(z, spec.act))
                if kind == "conv":
                    dW, db, da = L.conv2d_backward(dz, x_in, W_b[pi], spec.stride, spec.pad)
                else:
                    dW, db, da = L.dense_backward(dz, x_in, W_b[pi])
                g[pi] += dW
                g[pi + 1] += db
            dx_parts.append(self.q(da))
        self.g = g
        # the intermediate weights are built: this mini-batch no longer needs its stale version
        if self.policy not in ("latest", "timeprest"):
            self.refcnt[rec["v_f"]] -= 1
            self._evict_if_unused(rec["v_f"])
        del self.inflight[mb]
        return None if self.first_stage else np.concatenate(dx_parts, axis=0)

    # -- update ----------------------------------------------------------
    def update(self, mb: int) -> int:
        if self.g is None:
            raise StageError("update without a gradient")
        old = self.latest
        W = self.weights[old]
        new = []
        for i, (w, g) in enumerate(zip(W, self.g)):
            self.m[i] = self.mu * self.m[i] + g
            new.append(w - self.lr * self.m[i])
        self.latest = old + 1
        self.weights[self.latest] = new
        self.refcnt[self.latest] = 0
        self.g = None
        self.trace.append(("U", mb, old, self.latest, 0))
        self._evict_if_unused(old)                         # V: always; I: unless still stashed
        return self.latest

    def _evict_if_unused(self, v: int) -> None:
        if v != self.latest and v in self.weights and self.refcnt.get(v, 0) == 0:
            del self.weights[v]
            del self.refcnt[v]
            self.evicted.append(v)

    # -- inspection ------------------------------------------------------
    def live_versions(self) -> List[int]:
        return sorted(self.weights)

    def flat(self, plist: List[np.ndarray]) -> np.ndarray:
        return np.concatenate([p.reshape(-1) for p in plist])
