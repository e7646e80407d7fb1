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
