"""Runs DistFlashAttn schedules on one GPU with virtual workers.

Host-side sequencing only: which chunk pair is computed when comes from `dfa_schedule`
(Section 3.2, Algorithm 2), every computation is a call into libdfa.so.  "Sending" a
partial result to another worker is just handing over a buffer, since all P workers live
on the same device here.
"""
from __future__ import annotations

import torch

from . import binding as B


class Buffers:
    """Device buffers for one run, allocated once so that timed regions allocate nothing."""

    def __init__(self, h_q, h_kv, n, d, p, device, o_dtype=torch.float32, n_partials=1, grads=True, outputs=True):
        c = n // p
        self.c, self.p = c, p
        if outputs:     # False: the caller supplies O and L (a backward from saved tensors)
            self.O = torch.empty((h_q, n, d), dtype=o_dtype, device=device)
            self.L = torch.empty((h_q, n), dtype=torch.float32, device=device)
            self.part_o = [torch.empty((h_q, c, d), dtype=o_dtype, device=device) for _ in range(n_partials)]
            self.part_l = [torch.empty((h_q, c), dtype=torch.float32, device=device) for _ in range(n_partials)]
        if grads:
            self.delta = torch.empty((h_q, n), dtype=torch.float32, device=device)
            self.dQ = torch.zeros((h_q, n, d), dtype=torch.float32, device=device)
            self.dK = torch.zeros((h_kv, n, d), dtype=torch.float32, device=device)
            self.dV = torch.zeros((h_kv, n, d), dtype=torch.float32, device=device)


def _chunk(t, i, c):
    return t[:, i * c:(i + 1) * c]


class KVPrefetcher:
    """Emulates the overlap of Section 3.2 (Eq. 3) on one GPU: the key/value chunk a worker needs at
    step t + 1 is copied into a staging buffer on a second stream while step t computes.  The
    device-to-device copy stands in for the fetch from the peer that owns the chunk; the kernels of
    OWN pairs then read the staged copy, so the dependency (copy before use, use before the buffer is
    overwritten) is the real one.  Both streams have the default priority."""

    def __init__(self, K, V, c):
        self.K, self.V, self.c = K, V, c
        self.stream = torch.cuda.Stream()
        self.buf = [(torch.empty_like(K[:, :c]), torch.empty_like(V[:, :c])) for _ in range(2)]
        self.ev = [torch.cuda.Event(), torch.cuda.Event()]
        self.n = 0

    def fetch(self, kv_chunk):
        """Start copying chunk `kv_chunk` into the next staging slot; returns the slot."""
        slot = self.n & 1
        self.n += 1
        # the slot's previous readers (kernels already queued on the compute stream) come first
        self.stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(self.stream):
            self.buf[slot][0].copy_(_chunk(self.K, kv_chunk, self.c), non_blocking=True)
            self.buf[slot][1].copy_(_chunk(self.V, kv_chunk, self.c), non_blocking=True)
            self.ev[slot].record()
        return slot

    def get(self, slot):
        torch.cuda.current_stream().wait_event(self.ev[slot])
        return self.buf[slot]


def _own_steps(sched):
    return [st for st in sched if st.kind == B.DFA_STEP_OWN]


def forward_worker(Q, K, V, scale, P, w, bufs: Buffers, remote=None, mode="balanced", fused=True, prefetch=None):
    """Forward share of worker w: its diagonal chunk, its OWN pairs folded into (O_w, L_w),
    the partials that arrive from helpers (`remote`: {helper_id: (o, lse)}) merged at the step
    they arrive, and its HELP pairs computed into fresh partial buffers.
    fused: OWN pairs continue from the state in (O_w, L_w) (dfa_chunk_fwd_acc, the attn(q, k, v,
    o, s) call of Algorithms 1-2); otherwise each is a partial result plus a dfa_merge.
    prefetch: a KVPrefetcher; the key/value chunk of every OWN pair is then staged one step ahead
    on a second stream (fused path only).
    Returns {owner_id: (o_part, lse_part)} for the HELP pairs this worker computed."""
    c = bufs.c
    sent = {}
    o_w, l_w = _chunk(bufs.O, w, c), _chunk(bufs.L, w, c)
    sched = B.dfa_schedule(P, w, mode)
    own = _own_steps(sched) if prefetch is not None else []
    nxt, slot = 0, None
    for st in sched:
        if st.kind == B.DFA_STEP_DIAG:
            if own:
                slot = prefetch.fetch(own[0].kv_chunk); nxt = 1      # copy for step 1 runs under the diagonal pair
            B.dfa_chunk_fwd(_chunk(Q, w, c), _chunk(K, w, c), _chunk(V, w, c), True, scale, o=o_w, lse=l_w)
        elif st.kind == B.DFA_STEP_OWN and fused and prefetch is not None:
            k_s, v_s = prefetch.get(slot)
            if nxt < len(own):
                slot = prefetch.fetch(own[nxt].kv_chunk); nxt += 1   # copy for the next step runs under this pair
            B.dfa_chunk_fwd_acc(_chunk(Q, w, c), k_s, v_s, False, scale, o_w, l_w)
        elif st.kind == B.DFA_STEP_OWN and fused:
            B.dfa_chunk_fwd_acc(_chunk(Q, w, c), _chunk(K, st.kv_chunk, c), _chunk(V, st.kv_chunk, c), False, scale,
                                o_w, l_w)
        elif st.kind == B.DFA_STEP_OWN:
            po, pl = bufs.part_o[0], bufs.part_l[0]
            B.dfa_chunk_fwd(_chunk(Q, w, c), _chunk(K, st.kv_chunk, c), _chunk(V, st.kv_chunk, c), False, scale,
                            o=po, lse=pl)
            B.dfa_merge(o_w, l_w, po, pl)
        elif st.kind == B.DFA_STEP_HELP:
            po = torch.empty_like(bufs.part_o[0]); pl = torch.empty_like(bufs.part_l[0])
            B.dfa_chunk_fwd(_chunk(Q, st.q_chunk, c), _chunk(K, w, c), _chunk(V, w, c), False, scale, o=po, lse=pl)
            sent[st.send_to] = (po, pl)
        if st.recv_from >= 0 and remote is not None:
            ro, rl = remote[st.recv_from]
            B.dfa_merge(o_w, l_w, ro, rl)
    return sent


def new_pass():
    """Bookkeeping of one backward pass: which dQ / dK,dV chunks already hold a contribution.
    The first contribution to a chunk overwrites it (no zero-fill, no read of stale values), the
    later ones accumulate."""
    return {"dq": set(), "dkv": set()}


def backward_worker(Q, K, V, dO, scale, P, w, bufs: Buffers, mode="balanced", with_delta=True, touched=None):
    """Backward of the pairs worker w computed in the forward (same pair -> worker assignment),
    from the final merged O and L of each query chunk; nothing of the forward is re-run.
    For a HELP pair the logsumexp and D of the helped chunk must already be in `bufs`
    (in the distributed setting they travel with that chunk's queries and dO).
    touched: a new_pass() record shared by the calls of one pass; None = always accumulate into
    what the gradient buffers hold."""
    c = bufs.c
    for st in B.dfa_schedule(P, w, mode):
        if st.kind == B.DFA_STEP_IDLE:
            continue
        qc, kc = st.q_chunk, st.kv_chunk
        if with_delta and st.kind == B.DFA_STEP_DIAG:
            B.dfa_delta(_chunk(bufs.O, qc, c), _chunk(dO, qc, c), delta=_chunk(bufs.delta, qc, c))
        args = (_chunk(Q, qc, c), _chunk(K, kc, c), _chunk(V, kc, c), _chunk(bufs.L, qc, c),
                _chunk(bufs.delta, qc, c), _chunk(dO, qc, c))
        diag = st.kind == B.DFA_STEP_DIAG
        acc_q = touched is None or qc in touched["dq"]
        acc_kv = touched is None or kc in touched["dkv"]
        if acc_q == acc_kv:
            B.dfa_chunk_bwd(*args, _chunk(bufs.dQ, qc, c), _chunk(bufs.dK, kc, c), _chunk(bufs.dV, kc, c), diag, scale,
                            accumulate=acc_q)
        else:   # one side starts fresh, the other accumulates: the two halves of the call, one after the other
            B.dfa_chunk_bwd(*args, None, _chunk(bufs.dK, kc, c), _chunk(bufs.dV, kc, c), diag, scale, accumulate=acc_kv)
            B.dfa_chunk_bwd(*args, _chunk(bufs.dQ, qc, c), None, None, diag, scale, accumulate=acc_q)
        if touched is not None:
            touched["dq"].add(qc); touched["dkv"].add(kc)


def run_worker_share(Q, K, V, dO, scale, P, w, bufs: Buffers, remote, fused=True):
    """One pass of worker w's whole share: forward (incl. merges of the helpers' partials),
    the D pre-pass and the backward of the same pairs.  The gradient chunks the share touches are
    overwritten with the share's own sums (first contribution overwrites, the rest accumulate)."""
    forward_worker(Q, K, V, scale, P, w, bufs, remote=remote, fused=fused)
    backward_worker(Q, K, V, dO, scale, P, w, bufs, touched=new_pass())


def helper_partials_for(Q, K, V, scale, P, w, bufs: Buffers):
    """The partial results other workers compute for worker w's queries under the balanced
    schedule (what arrives over the network in the distributed setting)."""
    c = bufs.c
    out = {}
    for st in B.dfa_schedule(P, w):
        if st.recv_from >= 0:
            h = st.recv_from
            po = torch.empty_like(bufs.part_o[0]); pl = torch.empty_like(bufs.part_l[0])
            B.dfa_chunk_fwd(_chunk(Q, w, c), _chunk(K, h, c), _chunk(V, h, c), False, scale, o=po, lse=pl)
            out[h] = (po, pl)
    return out


def run_all_workers(Q, K, V, dO, scale, P, bufs: Buffers, mode="balanced", backward=True, fused=True):
    """The whole schedule of all P workers, time step by time step, on one GPU.
    fused: OWN pairs continue from the owner's state (dfa_chunk_fwd_acc) instead of partial + merge."""
    c = bufs.c
    scheds = [B.dfa_schedule(P, w, mode) for w in range(P)]
    nsteps = len(scheds[0])
    for t in range(nsteps):
        arrivals = []
        for w in range(P):
            st = scheds[w][t]
            if st.kind == B.DFA_STEP_DIAG:
                B.dfa_chunk_fwd(_chunk(Q, w, c), _chunk(K, w, c), _chunk(V, w, c), True, scale,
                                o=_chunk(bufs.O, w, c), lse=_chunk(bufs.L, w, c))
            elif st.kind == B.DFA_STEP_OWN and fused:
                B.dfa_chunk_fwd_acc(_chunk(Q, w, c), _chunk(K, st.kv_chunk, c), _chunk(V, st.kv_chunk, c), False,
                                    scale, _chunk(bufs.O, w, c), _chunk(bufs.L, w, c))
            elif st.kind == B.DFA_STEP_OWN:
                po, pl = bufs.part_o[0], bufs.part_l[0]
                B.dfa_chunk_fwd(_chunk(Q, w, c), _chunk(K, st.kv_chunk, c), _chunk(V, st.kv_chunk, c), False,
                                scale, o=po, lse=pl)
                B.dfa_merge(_chunk(bufs.O, w, c), _chunk(bufs.L, w, c), po, pl)
            elif st.kind == B.DFA_STEP_HELP:
                po, pl = bufs.part_o[0], bufs.part_l[0]
                B.dfa_chunk_fwd(_chunk(Q, st.q_chunk, c), _chunk(K, w, c), _chunk(V, w, c), False, scale,
                                o=po, lse=pl)
                # "send": the owner merges it in this same step
                B.dfa_merge(_chunk(bufs.O, st.send_to, c), _chunk(bufs.L, st.send_to, c), po, pl)
                arrivals.append((st.send_to, w))
        for owner, helper in arrivals:
            assert scheds[owner][t].recv_from == helper
    if backward:
        # a helper's backward needs D of the chunk it helped, so all D vectors come first
        for w in range(P):
            B.dfa_delta(_chunk(bufs.O, w, c), _chunk(dO, w, c), delta=_chunk(bufs.delta, w, c))
        touched = new_pass()
        for w in range(P):
            backward_worker(Q, K, V, dO, scale, P, w, bufs, mode, with_delta=False, touched=touched)
