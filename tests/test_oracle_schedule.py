"""Pins for oracle/schedule.py: the numbers and closed forms the paper prints, and
brute-force coverage invariants (each causal chunk pair exactly once)."""
import os
from fractions import Fraction

import pytest

from oracle import schedule as S

GOLD = os.path.join(os.path.dirname(__file__), "golden", "schedule_paper_values.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = [x.strip() for x in line.split("=")]
            out[k] = float(v)
    return out


def test_paper_printed_values_p8():
    g = _gold()
    P = int(g["P"])
    bal, ring = S.balanced(P), S.ring(P)
    # Section 4.5: 36 units of work in total, for either schedule
    assert len(S.pairs(bal)) == g["total_work_units"]
    assert len(S.pairs(ring)) == g["total_work_units"]
    # ring: 8 steps, capacity 64 -> 4.5x ; balanced: 5 steps -> 7.2x
    assert all(len(w) == g["ring_time_steps"] for w in ring)
    assert P * len(ring[0]) == g["ring_capacity_units"]
    assert g["total_work_units"] / len(ring[0]) == g["ring_expected_speedup"]
    assert all(len(w) == 1 + P // 2 for w in bal)
    assert g["total_work_units"] / len(bal[0]) == pytest.approx(g["balanced_expected_speedup"])


@pytest.mark.parametrize("P", list(range(1, 34)) + [64])
def test_idle_fraction_closed_forms(P):
    # Section 3.2: denominators are the P^2 slots of the unbalanced schedule
    ring, bal = S.ring(P), S.balanced(P)
    assert Fraction(S.idle_slots(ring), P * P) == Fraction(P * P - P, 2 * P * P)
    expect = Fraction(1, 2 * P) if P % 2 == 0 else Fraction(0)
    assert Fraction(S.idle_slots(bal), P * P) == expect


@pytest.mark.parametrize("P", list(range(1, 34)) + [64])
def test_every_causal_pair_exactly_once(P):
    want = sorted((p, r) for p in range(P) for r in range(p + 1))
    assert sorted(S.pairs(S.balanced(P))) == want
    assert sorted(S.pairs(S.ring(P))) == want


@pytest.mark.parametrize("P", list(range(1, 20)))
def test_balanced_structure(P):
    bal = S.balanced(P)
    for w, steps in enumerate(bal):
        assert steps[0]["kind"] == S.DIAG and steps[0]["q_chunk"] == w == steps[0]["kv_chunk"]
        for st in steps[1:]:
            t = st["t"]
            if st["kind"] == S.OWN:
                assert st["q_chunk"] == w and st["kv_chunk"] == w - t
            elif st["kind"] == S.HELP:
                # helper uses its own keys/values and another worker's queries, at distance P - t
                assert st["kv_chunk"] == w and st["q_chunk"] - w == P - t
                owner = st["send_to"]
                assert owner == st["q_chunk"]
                assert bal[owner][t]["recv_from"] == w
            if st["recv_from"] >= 0:
                h = st["recv_from"]
                assert bal[h][t]["kind"] == S.HELP and bal[h][t]["send_to"] == w


def test_tables_p4():
    # hand-derived from Algorithm 2 for P=4 (0-indexed): rows = workers, columns t=0..2
    bal = S.balanced(4)
    kinds = [[s["kind"] for s in w] for w in bal]
    assert kinds == [[S.DIAG, S.HELP, S.IDLE], [S.DIAG, S.OWN, S.IDLE],
                     [S.DIAG, S.OWN, S.OWN], [S.DIAG, S.OWN, S.OWN]]
    assert (bal[0][1]["q_chunk"], bal[0][1]["kv_chunk"]) == (3, 0)
    assert bal[3][1]["recv_from"] == 0 and bal[3][2]["recv_from"] == -1


@pytest.mark.parametrize("P,W", [(8, 1), (8, 3), (5, 0), (4, 7)])
def test_window_schedule(P, W):
    """Local sliding window (appendix on sparse patterns): worker w computes the pairs with the
    min(w, W) preceding chunks and nothing else; the appendix's example (P = 8, window of one
    worker: worker 7 attends to itself and worker 6) is the (8, 1) case."""
    sched = S.window(P, W)
    want = sorted((p, r) for p in range(P) for r in range(max(0, p - W), p + 1))
    assert sorted(S.pairs(sched)) == want
    assert all(len(w) == 1 + min(W, P - 1) for w in sched)
    assert all(s["kind"] != S.HELP for w in sched for s in w)
    if (P, W) == (8, 1):
        assert [(s["q_chunk"], s["kv_chunk"]) for s in sched[7]] == [(7, 7), (7, 6)]
