"""K stages driven through the nF1B event order on one host (fp64).

The activations a stage hands to the next one and the gradients it hands
back are plain arrays here; the order of events is the one `schedule.simulate`
produces (Section "Methodology").  The last stage takes the softmax
cross-entropy loss, averaged over the whole mini-batch, and starts the
backward pass.
"""
from __future__ import annotations

from typing import Callable, Dict, List

import numpy as np

from . import layers as L
from .schedule import simulate
from .stage import Stage


class Pipeline:
    def __init__(self, stage_specs, stage_params, *, policy, lam, lr, momentum, n, mb):
        self.K = len(stage_specs)
        self.n, self.mb = n, mb
        self.stages = [Stage(stage_specs[s], stage_params[s], policy=policy, lam=lam, lr=lr,
                             momentum=momentum, n=n, first_stage=(s == 0))
                       for s in range(self.K)]
        self.losses: Dict[int, float] = {}
        self.records: List[dict] = []

    def run(self, num_mb: int, get_input: Callable[[int], np.ndarray],
            get_labels: Callable[[int], np.ndarray], on_event=None):
        """Run num_mb mini-batches; `on_event(event, pipeline, info)` is called after each event."""
        events, table = simulate(self.K, num_mb)
        acts: Dict[tuple, np.ndarray] = {}      # (s, j) -> output of stage s for mini-batch j
        grads: Dict[tuple, np.ndarray] = {}     # (s, j) -> gradient w.r.t. the input of stage s
        for ev in events:
            s, j = ev.s, ev.j
            st = self.stages[s]
            info = {}
            if ev.kind == "F":
                x = get_input(j) if s == 0 else acts.pop((s - 1, j))
                outs = [st.forward(j, ub, x[ub * self.mb:(ub + 1) * self.mb]) for ub in range(self.n)]
                acts[(s, j)] = np.concatenate(outs, axis=0)
                info["y"] = acts[(s, j)]
                info["v_f"] = st.inflight[j]["v_f"]
            else:
                if s == self.K - 1:
                    logits = acts.pop((s, j))
                    loss, dlogits = L.softmax_cross_entropy(logits, get_labels(j), self.n * self.mb)
                    self.losses[j] = loss
                    dy = dlogits
                    info["loss"] = loss
                else:
                    dy = grads.pop((s + 1, j))
                info["dy"] = dy
                dx = st.backward(j, dy)
                if s > 0:
                    grads[(s, j)] = dx
                info["dx"] = dx
                info["g"] = st.flat(st.g)
                info["W_b"] = st.flat(st.last_W_b)
                info["trace"] = st.trace[-1]
                st.update(j)
                info["m"] = st.flat(st.m)
                info["W_new"] = st.flat(st.weights[st.latest])
                info["live"] = st.live_versions()
            if on_event is not None:
                on_event(ev, self, info)
        return events, table
