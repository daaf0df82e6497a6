"""Reference enumerator of the ring and load-balanced schedules.

TEST INFRASTRUCTURE ONLY (see the package docstring).  The schedules of Section 3.2 /
Appendix A of the DistFlashAttn paper, written out from what they assign rather than from the
printed per-worker listings: the causal chunk pairs are grouped by their DISTANCE
(query chunk minus key/value chunk), and each time step hands whole distance classes to
workers.  Workers and chunks are 0-indexed here, as in the library (the paper counts from 1).

Balanced schedule, P workers, time steps t = 0 .. floor(P/2):
* t = 0: every worker computes its own causal diagonal pair (distance 0).
* t >= 1: the pairs at distance t are (p, p - t) for p >= t; worker p computes its own (OWN).
  The t workers w < t have no pair at that distance.  Each of them holds the key/value chunk of
  exactly one pair at distance P - t, namely (w + P - t, w), whose owner is busy with its own
  distance-t pair: w computes it with the owner's queries (HELP) and sends the partial result
  to the owner, who merges it at this step.
* If P - t == t (P even, t = P/2) the distance-(P - t) pairs ARE the own pairs of this step, so
  nobody helps and the workers w < t idle.

Readings taken where the printed algorithm is ambiguous:
* Its guard "t != floor(P/2)" on the helper and receive branches is read as "2t != P": helper
  work is skipped only when both distances coincide.  With the printed guard an odd P would
  never compute the pairs at distance (P+1)/2, contradicting the stated idle fraction of 0 for
  odd P (Section 3.2).
* Its index (p - t) mod P of a 1-indexed worker yields 0 for worker P; the key/value fetched
  on the own branch is that worker's (the arrow label's subscript t is a typo).
"""
from __future__ import annotations

IDLE, DIAG, OWN, HELP = 0, 1, 2, 3


def _step(t, kind=IDLE, q_chunk=-1, kv_chunk=-1, send_to=-1, recv_from=-1):
    return dict(t=t, kind=kind, q_chunk=q_chunk, kv_chunk=kv_chunk, send_to=send_to, recv_from=recv_from)


def balanced(P: int):
    """Step lists of all P workers under the balanced schedule: out[w][t] is a dict with the fields
    t, kind, q_chunk, kv_chunk, send_to, recv_from (-1 where not applicable)."""
    assert P >= 1
    n_steps = 1 + P // 2
    out = [[_step(t) for t in range(n_steps)] for _ in range(P)]
    for w in range(P):
        out[w][0] = _step(0, DIAG, w, w)
    for t in range(1, n_steps):
        for p in range(t, P):                      # distance t: the owner of the queries computes it
            out[p][t] = _step(t, OWN, p, p - t)
        far = P - t                                # the distance handed to the workers without own work
        if far != t:
            for p in range(far, P):
                helper = p - far                   # holds the pair's key/value chunk, and is < t
                assert out[helper][t]["kind"] == IDLE
                out[helper][t] = _step(t, HELP, p, helper, send_to=p)
                out[p][t]["recv_from"] = helper
    return out


def balanced_worker(P: int, w: int):
    """Steps of (0-indexed) worker w under the balanced schedule."""
    assert 0 <= w < P
    return balanced(P)[w]


def ring_worker(P: int, w: int):
    """Steps of (0-indexed) worker w under the vanilla (unbalanced) schedule: the diagonal pair,
    then its pairs in order of growing distance, one per time step; P time steps in all, the
    worker idles once it has run out of earlier chunks."""
    assert 0 <= w < P
    return [_step(0, DIAG, w, w)] + [_step(t, OWN, w, w - t) if t <= w else _step(t) for t in range(1, P)]


def window_worker(P: int, w: int, window_chunks: int):
    """Steps of (0-indexed) worker w when attention is local to the `window_chunks` preceding
    chunks (appendix on sparse patterns, local sliding windows): the vanilla schedule cut off
    after distance `window_chunks`.  1 + min(window_chunks, P - 1) time steps; no helpers (the load
    is near balanced by itself)."""
    assert 0 <= w < P and window_chunks >= 0
    return ring_worker(P, w)[:1 + min(window_chunks, P - 1)]


def ring(P: int):
    return [ring_worker(P, w) for w in range(P)]


def window(P: int, window_chunks: int):
    return [window_worker(P, w, window_chunks) for w in range(P)]


def idle_slots(sched) -> int:
    return sum(1 for w in sched for s in w if s["kind"] == IDLE)


def pairs(sched):
    """All (q_chunk, kv_chunk) pairs computed anywhere in the schedule."""
    return [(s["q_chunk"], s["kv_chunk"]) for w in sched for s in w if s["kind"] != IDLE]
