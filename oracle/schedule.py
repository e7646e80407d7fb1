"""nF1B event order of a K-stage pipeline at mini-batch granularity.

Section "Methodology": every mini-batch is split into n micro-batches whose
forward passes run back to back at a stage, and one backward pass serves the
whole mini-batch; the weights are updated after every mini-batch.  The timing
diagrams themselves are not available, so the order is rebuilt from the
prose: stage s (0-indexed) takes in K - s mini-batches before its first
backward and then alternates {backward j, update j, forward of the next
mini-batch}.  This reproduces every version example the text gives
(Sections "Methodology", "V-TiMePReSt", "I-TiMePReSt").

Two independent statements of the same schedule live here: a discrete-time
simulation (`simulate`) and the closed form (`closed_form`).  Tests check one
against the other and both against the paper's worked examples.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple


@dataclass(frozen=True)
class Event:
    t: int        # time step
    kind: str     # "F" forward of all n micro-batches | "B" backward + update
    s: int        # stage
    j: int        # mini-batch


def closed_form(K: int, s: int, j: int) -> Tuple[int, int, int]:
    """(v_f, v_now, delta) of mini-batch j at stage s, all 0-indexed.

    v_f    version (number of updates applied) the forward pass reads
    v_now  latest version when the backward pass of j runs at stage s
    delta  v_now - v_f
    """
    lag = K - 1 - s
    v_f = max(0, j - lag)
    v_now = j
    return v_f, v_now, v_now - v_f


def simulate(K: int, num_mb: int) -> Tuple[List[Event], Dict[Tuple[int, int], Tuple[int, int, int]]]:
    """Run the pipeline clock and return (events in execution order, version table).

    Each stage owns a fixed list of operations: K-s forwards, then
    backward/forward alternating until all mini-batches are done.  At every
    time step a stage runs its next operation if the data it needs was
    produced at an earlier time step: a forward needs the previous stage's
    forward of the same mini-batch, a backward needs the next stage's backward
    (the last stage needs its own forward, after which it takes the loss).
    Within a time step backward events are listed from the last stage to the
    first, then forward events from the first stage to the last.
    """
    ops: List[List[Tuple[str, int]]] = []
    for s in range(K):
        warm = min(K - s, num_mb)
        seq = [("F", j) for j in range(warm)]
        nf, nb = warm, 0
        while nb < num_mb:
            seq.append(("B", nb)); nb += 1
            if nf < num_mb:
                seq.append(("F", nf)); nf += 1
        ops.append(seq)

    pos = [0] * K
    done_at: Dict[Tuple[str, int, int], int] = {}
    version = [0] * K                      # updates applied per stage
    table: Dict[Tuple[int, int], List[int]] = {}
    events: List[Event] = []
    t = 0
    while any(pos[s] < len(ops[s]) for s in range(K)):
        ready = []
        for s in range(K):
            if pos[s] >= len(ops[s]):
                continue
            kind, j = ops[s][pos[s]]
            if kind == "F":
                ok = s == 0 or done_at.get(("F", s - 1, j), t) < t
            else:
                dep = ("F", s, j) if s == K - 1 else ("B", s + 1, j)
                ok = done_at.get(dep, t) < t
            if ok:
                ready.append((kind, s, j))
        if not ready:
            raise RuntimeError("pipeline deadlock")
        order = sorted([e for e in ready if e[0] == "B"], key=lambda e: -e[1]) + \
                sorted([e for e in ready if e[0] == "F"], key=lambda e: e[1])
        for kind, s, j in order:
            if kind == "F":
                table[(s, j)] = [version[s], -1, -1]
            else:
                v_f = table[(s, j)][0]
                table[(s, j)] = [v_f, version[s], version[s] - v_f]
                version[s] += 1            # update after every mini-batch
            done_at[(kind, s, j)] = t
            pos[s] += 1
            events.append(Event(t, kind, s, j))
        t += 1
    return events, {k: tuple(v) for k, v in table.items()}


# ---------------------------------------------------------------------------
# Micro-batch granularity
# ---------------------------------------------------------------------------

@dataclass(frozen=True)
class MicroEvent:
    t: int        # time step
    kind: str     # "F" forward of ONE micro-batch | "B" backward of the mini-batch + update
    s: int        # stage
    j: int        # mini-batch
    ub: int       # micro-batch (0 for "B")
    version: int  # latest version at the stage when the event runs (before the update of a "B")


def simulate_microbatches(K: int, num_mb: int, n: int, mid_pass_updates: bool) -> List[MicroEvent]:
    """The pipeline clock with one box per stage and time step, a box being the forward pass of one micro-batch
    or the backward pass of one mini-batch (the way the paper's timing figures are described: Section
    "Methodology", last paragraph).  A stage takes the next micro-batch as soon as the previous stage has
    produced it, holds at most K - s mini-batches between their first forward and their backward, and gives a
    backward pass that is ready precedence over further forwards:

      mid_pass_updates = True   also between two micro-batches of one mini-batch -- the update then lands in
                                the middle of that mini-batch's forward pass at this stage, and its remaining
                                micro-batches read the newer weights.  Only V-TiMePReSt allows this (it "checks
                                for the newer versions of weights even during the execution of a pass", Section
                                "V-TiMePReSt", Challenge 1);
      mid_pass_updates = False  only between mini-batches: a mini-batch whose forward has started at a stage
                                finishes it on one version (what stashing a forward version needs).

    Within a time step backward events are listed from the last stage to the first, then forward events from
    the first stage to the last; an event sees what earlier time steps produced."""
    nf = [[0, 0] for _ in range(K)]        # next forward per stage: (mini-batch, micro-batch)
    nb = [0] * K                           # next backward per stage
    version = [0] * K
    f_done: Dict[Tuple[int, int, int], int] = {}
    b_done: Dict[Tuple[int, int], int] = {}
    events: List[MicroEvent] = []
    t = 0
    while any(nb[s] < num_mb for s in range(K)):
        run = []
        for s in range(K):
            if nb[s] >= num_mb:
                continue
            jb = nb[s]
            if s == K - 1:
                b_ready = f_done.get((s, jb, n - 1), t) < t
            else:
                b_ready = b_done.get((s + 1, jb), t) < t
            jf, ub = nf[s]
            f_ready = jf < num_mb and (s == 0 or f_done.get((s - 1, jf, ub), t) < t) and \
                (ub > 0 or jf - nb[s] < K - s)                      # a new mini-batch only below the in-flight limit
            mid_pass = ub > 0                                       # a mini-batch's forward is under way here
            if b_ready and (mid_pass_updates or not mid_pass or not f_ready):
                run.append(("B", s, jb, 0))
            elif f_ready:
                run.append(("F", s, jf, ub))
        if not run:
            raise RuntimeError("pipeline deadlock")
        order = sorted([e for e in run if e[0] == "B"], key=lambda e: -e[1]) + \
                sorted([e for e in run if e[0] == "F"], key=lambda e: e[1])
        for kind, s, j, ub in order:
            events.append(MicroEvent(t, kind, s, j, ub, version[s]))
            if kind == "F":
                f_done[(s, j, ub)] = t
                nf[s] = [j, ub + 1] if ub + 1 < n else [j + 1, 0]
            else:
                b_done[(s, j)] = t
                version[s] += 1
                nb[s] += 1
        t += 1
    return events
