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


def pass_versions(events, K: int):
    """Per mini-batch, the version every stage held at the moment its forward pass started (first micro-batch at
    stage 0) and at the moment its backward pass started (at the last stage): what TiMePReSt runs those passes on
    ("during a pass it cannot utilize updated weights", Section "V-TiMePReSt", Challenge 1)."""
    version = [0] * K
    fwd, bwd = {}, {}
    for e in events:
        if e.kind == "F" and e.s == 0 and e.ub == 0:
            fwd[e.j] = tuple(version)
        if e.kind == "B" and e.s == K - 1:
            bwd[e.j] = tuple(version)
        if e.kind == "B":
            version[e.s] += 1
    return fwd, bwd


def run_microbatches(pipe: Pipeline, num_mb: int, get_input, get_labels, *, mid_pass_updates: bool = False, on_event=None):
    """Drive `pipe` through the micro-batch-granular clock (schedule.simulate_microbatches).  Under the policy
    "timeprest" every pass reads, at each stage, the version that stage held when the pass started; those versions
    are pinned when the pass starts and released stage by stage as the pass leaves."""
    from .schedule import simulate_microbatches
    K, n, mb = pipe.K, pipe.n, pipe.mb
    events = simulate_microbatches(K, num_mb, n, mid_pass_updates)
    timeprest = pipe.stages[0].policy == "timeprest"
    fwd_v, bwd_v = pass_versions(events, K)
    acts: Dict[tuple, list] = {}            # (s, j) -> outputs of stage s, one per micro-batch
    grads: Dict[tuple, np.ndarray] = {}
    inputs: Dict[int, np.ndarray] = {}
    for ev in events:
        s, j = ev.s, ev.j
        st = pipe.stages[s]
        info = {}
        if ev.kind == "F":
            if timeprest and s == 0 and ev.ub == 0:            # the forward pass starts: its versions stay alive
                for r in range(K):
                    assert pipe.stages[r].latest == fwd_v[j][r]
                    pipe.stages[r].pin(fwd_v[j][r])
            if s == 0:
                if j not in inputs:
                    inputs[j] = get_input(j)
                x = inputs[j][ev.ub * mb:(ev.ub + 1) * mb]
            else:
                x = acts[(s - 1, j)][ev.ub]
            assert st.latest == ev.version
            y = st.forward(j, ev.ub, x, version=fwd_v[j][s]) if timeprest else st.forward(j, ev.ub, x)
            acts.setdefault((s, j), []).append(y)
            info.update(y=y, version=st.inflight[j]["versions"][-1])
            if ev.ub == n - 1:
                if s == 0:
                    inputs.pop(j)
                else:
                    acts.pop((s - 1, j))
                if timeprest:
                    st.unpin(fwd_v[j][s])
        else:
            if timeprest and s == K - 1:                       # the backward pass starts
                for r in range(K):
                    assert pipe.stages[r].latest == bwd_v[j][r]
                    pipe.stages[r].pin(bwd_v[j][r])
            if s == K - 1:
                logits = np.concatenate(acts.pop((s, j)), axis=0)
                loss, dy = L.softmax_cross_entropy(logits, get_labels(j), n * mb)
                pipe.losses[j] = loss
                info["loss"] = loss
            else:
                dy = grads.pop((s + 1, j))
            info["dy"] = dy
            dx = st.backward(j, dy, version=bwd_v[j][s]) if timeprest else st.backward(j, dy)
            if timeprest:
                st.unpin(bwd_v[j][s])
            if s > 0:
                grads[(s, j)] = dx
            info.update(dx=dx, g=st.flat(st.g), trace=st.trace[-1])
            st.update(j)
            info.update(m=st.flat(st.m), W_new=st.flat(st.weights[st.latest]))
        info["live"] = st.live_versions()
        info["refcnt"] = dict(st.refcnt)
        if on_event is not None:
            on_event(ev, pipe, info)
    return events, (fwd_v, bwd_v)
