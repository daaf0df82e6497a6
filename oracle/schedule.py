"""Reference enumerator of the ring and load-balanced schedules.

TEST INFRASTRUCTURE ONLY (see the package docstring).  It walks the two
per-worker algorithms of Appendix A of the DistFlashAttn paper (vanilla and
balanced) in the paper's own 1-indexed notation, step by step, and only at the
end converts worker/chunk numbers to the 0-indexed ones the library uses.

Readings taken where the printed algorithm is ambiguous:
* r = (p - t) mod P is a 1-indexed worker, so a result of 0 denotes worker P.
* The guard printed as "t != floor(P/2)" on the helper and receive branches is
  read as "2t != P": the helper work at distance P - t is skipped only when it
  coincides with the own work at distance t (P even, t = P/2).  With the printed
  guard an odd P would drop pairs, contradicting the stated idle fraction of 0
  for odd P (Section 3.2).
* The key/value fetched on the own branch is k_r, v_r (the arrow label's
  subscript t is a typo).
"""
from __future__ import annotations

IDLE, DIAG, OWN, HELP = 0, 1, 2, 3


def _wrap(x: int, P: int) -> int:
    """1-indexed modulo: maps 0 to P."""
    x %= P
    return P if x == 0 else x


def balanced_worker(P: int, p1: int):
    """Steps of 1-indexed worker p1 under the balanced algorithm.

    Returns a list of dicts with 0-indexed fields:
    t, kind, q_chunk, kv_chunk, send_to, recv_from  (-1 where not applicable).
    """
    assert 1 <= p1 <= P
    steps = [dict(t=0, kind=DIAG, q_chunk=p1 - 1, kv_chunk=p1 - 1, send_to=-1, recv_from=-1)]
    for t in range(1, P // 2 + 1):
        r = _wrap(p1 - t, P)
        st = dict(t=t, kind=IDLE, q_chunk=-1, kv_chunk=-1, send_to=-1, recv_from=-1)
        if p1 > t:
            # own work: my queries against the chunk t positions earlier
            st.update(kind=OWN, q_chunk=p1 - 1, kv_chunk=r - 1)
            if 2 * t != P and p1 + t > P:
                r2 = _wrap(p1 + t, P)
                st.update(recv_from=r2 - 1)
        else:
            if 2 * t != P:
                # helper: worker r's queries against my own keys/values
                st.update(kind=HELP, q_chunk=r - 1, kv_chunk=p1 - 1, send_to=r - 1)
        steps.append(st)
    return steps


def ring_worker(P: int, p1: int):
    """Steps of 1-indexed worker p1 under the vanilla (unbalanced) algorithm:
    diagonal first, then the chunks 1..p-1 positions earlier; P time steps in all,
    the worker idles once its own list is exhausted."""
    assert 1 <= p1 <= P
    steps = [dict(t=0, kind=DIAG, q_chunk=p1 - 1, kv_chunk=p1 - 1, send_to=-1, recv_from=-1)]
    for t in range(1, P):
        if t < p1:
            r = _wrap(p1 - t, P)
            steps.append(dict(t=t, kind=OWN, q_chunk=p1 - 1, kv_chunk=r - 1, send_to=-1, recv_from=-1))
        else:
            steps.append(dict(t=t, kind=IDLE, q_chunk=-1, kv_chunk=-1, send_to=-1, recv_from=-1))
    return steps


def window_worker(P: int, p1: int, window_chunks: int):
    """Steps of 1-indexed worker p1 when attention is local to the `window_chunks` preceding
    workers (appendix on sparse patterns, "local sliding windows"): the vanilla algorithm with
    the end of its loop moved from the first worker to the one `window_chunks` positions
    earlier.  1 + window_chunks time steps; no helpers (the load is near balanced by itself)."""
    assert 1 <= p1 <= P and window_chunks >= 0
    return ring_worker(P, p1)[:1 + min(window_chunks, P - 1)]


def balanced(P: int):
    """Step lists of all workers, 0-indexed by worker."""
    return [balanced_worker(P, p1) for p1 in range(1, P + 1)]


def ring(P: int):
    return [ring_worker(P, p1) for p1 in range(1, P + 1)]


def window(P: int, window_chunks: int):
    return [window_worker(P, p1, window_chunks) for p1 in range(1, P + 1)]


def idle_slots(sched) -> int:
    return sum(1 for w in sched for s in w if s["kind"] == IDLE)


def pairs(sched):
    """All (q_chunk, kv_chunk) pairs computed anywhere in the schedule."""
    return [(s["q_chunk"], s["kv_chunk"]) for w in sched for s in w if s["kind"] != IDLE]
