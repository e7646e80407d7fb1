"""Pins for the schedule: the paper's worked version examples, closed form vs simulation."""
import os

import pytest

from oracle.schedule import closed_form, simulate

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_version_examples.txt")


def _golden_lines():
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                yield line.split()


def test_paper_worked_examples_simulation_and_closed_form():
    K = 4
    _, table = simulate(K, 8)
    checked = 0
    for tok in _golden_lines():
        kind, args = tok[0], [int(t) for t in tok[1:]]
        if kind == "fwd":
            mb, stage, ver = args
            assert table[(stage - 1, mb - 1)][0] == ver
            assert closed_form(K, stage - 1, mb - 1)[0] == ver
        elif kind == "bwd":
            mb, stage, stale, latest = args
            assert table[(stage - 1, mb - 1)][:2] == (stale, latest)
            assert closed_form(K, stage - 1, mb - 1)[:2] == (stale, latest)
        elif kind in ("same", "diff"):
            mb, sa, sb = args
            va, vb = table[(sa - 1, mb - 1)][0], table[(sb - 1, mb - 1)][0]
            assert (va == vb) == (kind == "same")
        else:
            raise AssertionError(tok)
        checked += 1
    assert checked == 19


@pytest.mark.parametrize("K", [1, 2, 3, 4, 6])
def test_simulation_equals_closed_form(K):
    num = 12
    events, table = simulate(K, num)
    assert len(table) == K * num
    for (s, j), triple in table.items():
        assert triple == closed_form(K, s, j)
        assert triple[2] == min(j, K - 1 - s)          # degree of staleness
    # every mini-batch passes every stage exactly once each way
    assert sorted((e.kind, e.s, e.j) for e in events) == sorted(
        (k, s, j) for k in "FB" for s in range(K) for j in range(num))


@pytest.mark.parametrize("K", [2, 4])
def test_event_order_respects_dependencies(K):
    events, _ = simulate(K, 9)
    seen = set()
    for e in events:
        if e.kind == "F" and e.s > 0:
            assert ("F", e.s - 1, e.j) in seen
        if e.kind == "B":
            assert ("F", e.s, e.j) in seen
            if e.s < K - 1:
                assert ("B", e.s + 1, e.j) in seen
        seen.add((e.kind, e.s, e.j))
    # the last stage never runs on stale weights; the first stage reaches staleness K-1
    _, table = simulate(K, 9)
    assert all(table[(K - 1, j)][2] == 0 for j in range(9))
    assert max(table[(0, j)][2] for j in range(9)) == K - 1


def test_in_flight_bound():
    # stage s never holds more than K - s mini-batches between forward and backward
    K = 4
    events, _ = simulate(K, 10)
    live = [0] * K
    for e in events:
        live[e.s] += 1 if e.kind == "F" else -1
        assert 0 <= live[e.s] <= K - e.s
    assert live == [0] * K


# ---- micro-batch granularity -------------------------------------------------------------------------------

from oracle.schedule import simulate_microbatches  # noqa: E402
from oracle.pipeline import pass_versions  # noqa: E402


def _forward_versions(events):
    tab = {}
    for e in events:
        if e.kind == "F":
            tab.setdefault((e.s, e.j), []).append(e.version)
    return tab


@pytest.mark.parametrize("K", [1, 2, 3, 4, 6])
@pytest.mark.parametrize("n", [1, 2, 4, 8])
def test_microbatch_clock_without_mid_pass_updates_is_the_minibatch_schedule(K, n):
    # every micro-batch of a mini-batch reads one version, and it is the closed form's (hence the paper's examples)
    num = 11
    events = simulate_microbatches(K, num, n, False)
    tab = _forward_versions(events)
    assert len(tab) == K * num
    for (s, j), versions in tab.items():
        assert len(versions) == n and len(set(versions)) == 1
        assert versions[0] == closed_form(K, s, j)[0]
    for e in events:
        if e.kind == "B":
            assert e.version == closed_form(K, e.s, e.j)[1]           # latest at the backward = j updates
    assert sum(e.kind == "F" for e in events) == K * num * n and sum(e.kind == "B" for e in events) == K * num


@pytest.mark.parametrize("mid", [False, True])
def test_microbatch_clock_reproduces_the_papers_examples_with_two_micro_batches(mid):
    # the paper's figures split every mini-batch into two micro-batches on four workers: all its version examples
    # hold at micro-batch granularity, with and without updates allowed in the middle of a pass
    tab = _forward_versions(simulate_microbatches(4, 8, 2, mid))
    bwd = {(e.s, e.j): e.version for e in simulate_microbatches(4, 8, 2, mid) if e.kind == "B"}
    checked = 0
    for tok in _golden_lines():
        kind, args = tok[0], [int(t) for t in tok[1:]]
        if kind == "fwd":
            mb, stage, ver = args
            assert set(tab[(stage - 1, mb - 1)]) == {ver}
        elif kind == "bwd":
            mb, stage, stale, latest = args
            assert tab[(stage - 1, mb - 1)][0] == stale and bwd[(stage - 1, mb - 1)] == latest
        else:
            mb, sa, sb = args
            assert (tab[(sa - 1, mb - 1)] == tab[(sb - 1, mb - 1)]) == (kind == "same")
        checked += 1
    assert checked == 19


def test_an_update_lands_between_micro_batches_only_when_allowed():
    K, num, n = 4, 10, 4
    strict = _forward_versions(simulate_microbatches(K, num, n, False))
    loose = _forward_versions(simulate_microbatches(K, num, n, True))
    assert all(len(set(v)) == 1 for v in strict.values())
    split = {k: v for k, v in loose.items() if len(set(v)) > 1}
    assert split                                                     # it does happen ...
    for (s, j), v in loose.items():
        assert v == sorted(v)                                        # ... versions only move forward within a pass
        assert v[0] >= strict[(s, j)][0]                             # and are never older than without it
    # same amount of work, same number of time steps per stage either way
    for mid in (False, True):
        ev = simulate_microbatches(K, num, n, mid)
        for s in range(K):
            ticks = [e.t for e in ev if e.s == s]
            assert len(ticks) == len(set(ticks)) == num * (n + 1)    # one box per stage and time step


@pytest.mark.parametrize("mid", [False, True])
def test_microbatch_clock_respects_dependencies_and_in_flight_bound(mid):
    K, num, n = 4, 9, 4
    events = simulate_microbatches(K, num, n, mid)
    done = {}
    first_f, live = {}, [0] * K
    for e in events:
        if e.kind == "F":
            if e.s > 0:
                assert done[("F", e.s - 1, e.j, e.ub)] < e.t
            if e.ub > 0:
                assert done[("F", e.s, e.j, e.ub - 1)] < e.t
            else:
                live[e.s] += 1
                assert live[e.s] <= K - e.s
            done[("F", e.s, e.j, e.ub)] = e.t
        else:
            assert done[("F", e.s, e.j, n - 1)] < e.t
            if e.s < K - 1:
                assert done[("B", e.s + 1, e.j)] < e.t
            done[("B", e.s, e.j)] = e.t
            live[e.s] -= 1
    assert live == [0] * K


def test_timeprest_pass_versions():
    # TiMePReSt: every stage of a pass reads the version it held when the pass started.  The paper's remark (Section
    # "Methodology"): while the forward of mini-batch 4 moves from stage 1 to stage 2 the update of mini-batch 1 has
    # happened there; the version the pass started on is stale but still the one TiMePReSt uses -- V-TiMePReSt reads
    # the newer one.
    K, n = 4, 2
    events = simulate_microbatches(K, 8, n, False)
    fwd, bwd = pass_versions(events, K)
    v_tab = _forward_versions(events)
    assert fwd[3][1] == 0 and v_tab[(1, 3)][0] == 1
    for j in range(8):
        # recomputed independently: updates each stage had applied before the pass's first event
        t_f = next(i for i, e in enumerate(events) if e.kind == "F" and e.s == 0 and e.j == j and e.ub == 0)
        t_b = next(i for i, e in enumerate(events) if e.kind == "B" and e.s == K - 1 and e.j == j)
        for s in range(K):
            assert fwd[j][s] == sum(1 for e in events[:t_f] if e.kind == "B" and e.s == s)
            assert bwd[j][s] == sum(1 for e in events[:t_b] if e.kind == "B" and e.s == s)
            assert fwd[j][s] <= v_tab[(s, j)][0]                     # never newer than what V-TiMePReSt reads there
            assert bwd[j][s] <= j                                    # nor than the latest when the backward arrives
        assert fwd[j][0] == v_tab[(0, j)][0] and bwd[j][K - 1] == j  # equal where the pass starts
        assert fwd[j] != bwd[j] or j == 0                            # no horizontal stashing: the two passes differ
