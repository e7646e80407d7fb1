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
