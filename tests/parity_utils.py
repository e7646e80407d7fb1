"""Shared helpers of the GPU parity tests: run the oracle and the HIP library on the same
seeded inputs, event by event, and compare tensors and integer tables."""
from __future__ import annotations

import numpy as np

from oracle.pipeline import Pipeline
from synth_inputs import workloads as W

# relative Frobenius error allowed between the HIP path and the fp64 oracle
TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values from the GPU"
    denom = np.linalg.norm(ref)
    if denom == 0.0:
        return float(np.linalg.norm(got))
    return float(np.linalg.norm(got - ref) / denom)


def to_np(t):
    import torch
    return t.detach().to(torch.float64).cpu().numpy()


def oracle_records(w: W.Workload, policy: str, num_mb: int, params=None):
    """Run the oracle pipeline and keep everything each event produced."""
    params = params if params is not None else [W.init_params(w, s) for s in range(w.K)]
    pipe = Pipeline(w.stages, params, policy=policy, lam=w.lam, lr=w.lr, momentum=w.momentum, n=w.n, mb=w.mb)
    rec = {}

    def on_event(ev, p, info):
        st = p.stages[ev.s]
        keep = dict(info)
        if ev.kind == "B":
            gsq = float(np.sum(info["g"] ** 2))
            keep["diag_grad_sq"] = gsq
            keep["diag_weight_sq"] = float(np.sum(info["W_new"] ** 2))
        keep["latest"] = st.latest
        keep["live"] = st.live_versions()
        keep["refcnt"] = dict(st.refcnt)
        rec[(ev.kind, ev.s, ev.j)] = keep

    events, table = pipe.run(num_mb, lambda j: W.minibatch_input(w, j), lambda j: W.minibatch_labels(w, j),
                             on_event=on_event)
    return rec, events, table, pipe


def oracle_flat_to_arena(stage, flat_oracle: np.ndarray) -> np.ndarray:
    """Oracle's concatenated [W0,b0,W1,b1,...] -> the library's padded arena order."""
    from paper_2509_23241_amd.binding import layer_param_shapes
    parts, off = [], 0
    for spec in stage.layers:
        for shape in layer_param_shapes(spec):
            n = int(np.prod(shape))
            parts.append(flat_oracle[off: off + n].reshape(shape))
            off += n
    return stage.pack(parts).astype(np.float64)
