"""GPU parity, element by element against the fp64 oracle, at sizes the oracle finishes in
seconds: the merge, the D pre-pass, single chunk pairs (square, ragged, GQA, causal and
not), empty inputs, and whole balanced schedules incl. config 1."""
import math

import numpy as np
import pytest
import torch

import dfa_inputs
import paper_2310_03294_amd as dfa
from paper_2310_03294_amd import driver
from oracle import attention as A
from gpu_util import TOL, case, dev, maxerr, np64

pytestmark = pytest.mark.gpu


def _pair_oracle(q, k, v, do, scale, causal):
    """Expected (O, L, dq, dk, dv) of ONE pair used as a whole problem (its lse is the final one):
    the oracle's monolithic forward and analytic backward, causal for a square diagonal chunk,
    unmasked (any s_q, s_k) for an earlier chunk."""
    q64, k64, v64, do64 = (np64(t) for t in (q, k, v, do))
    O, L = A.attention_fwd(q64, k64, v64, scale, causal=causal)
    dq, dk, dv = A.attention_bwd(q64, k64, v64, do64, scale, causal=causal)
    return O, L, dq, dk, dv


SHAPES_F32 = [
    # h_q, h_kv, s_q, s_k, d, causal
    (1, 1, 256, 256, 64, True), (2, 2, 64, 64, 128, False), (4, 2, 130, 130, 64, True),
    (3, 1, 100, 77, 128, False), (2, 1, 1, 1, 64, True), (2, 2, 65, 191, 64, False), (8, 2, 257, 257, 128, True),
]
SHAPES_BF16 = [
    (2, 2, 128, 128, 128, True), (2, 2, 256, 192, 128, False), (4, 2, 384, 384, 128, True),
    (3, 1, 100, 77, 128, False), (2, 1, 1, 1, 128, True), (2, 2, 65, 191, 128, False), (8, 2, 257, 257, 128, True),
    (1, 1, 1024, 1024, 128, True), (2, 1, 640, 1152, 128, False),
    (4, 2, 333, 451, 128, False), (4, 2, 333, 333, 128, True),      # several tiles, ragged ends on both axes, grouped heads
    (64, 16, 4100, 333, 128, False),    # enough (head, 256-row tile) items for the 256-row dq workgroups, ragged
]


def _run_pair(dtype, h_q, h_kv, s_q, s_k, d, causal, o_dtype=torch.float32):
    q, k, v, do = case(1000 + s_q + s_k, h_q, h_kv, s_q, s_k, d, dtype)
    scale = 1 / math.sqrt(d)
    Q, K, V, dO = (t.to(dev()) for t in (q, k, v, do))
    o, lse = dfa.dfa_chunk_fwd(Q, K, V, causal, scale, o_dtype=o_dtype)
    delta = dfa.dfa_delta(o, dO)
    dq = torch.full((h_q, s_q, d), 7.0, device=dev()); dk = torch.full((h_kv, s_k, d), 7.0, device=dev())
    dv = torch.full((h_kv, s_k, d), 7.0, device=dev())
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, causal, scale, accumulate=False)
    torch.cuda.synchronize()
    O, L, rq, rk, rv = _pair_oracle(q, k, v, do, scale, causal)
    tol = TOL[dtype]
    errs = dict(o=maxerr(o, O), lse=maxerr(lse, L), dq=maxerr(dq, rq), dk=maxerr(dk, rk), dv=maxerr(dv, rv))
    assert all(e <= tol for e in errs.values()), errs
    # the D pre-pass against the oracle's on the same input (the o it was given); fp32 accumulation of d terms
    assert maxerr(delta, A.delta_rows(np64(o), np64(do))) <= 1e-4
    # accumulate != 0 adds the same contribution on top
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, causal, scale, accumulate=True)
    torch.cuda.synchronize()
    errs2 = dict(dq=maxerr(dq, 2 * rq), dk=maxerr(dk, 2 * rk), dv=maxerr(dv, 2 * rv))
    assert all(e <= 2 * tol for e in errs2.values()), errs2
    # a NULL output selects the other gradients only: (dk, dv) alone, then dq alone
    dq3 = torch.full_like(dq, 7.0); dk3 = torch.full_like(dk, 7.0); dv3 = torch.full_like(dv, 7.0)
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, None, dk3, dv3, causal, scale, accumulate=False)
    torch.cuda.synchronize()
    assert maxerr(dk3, rk) <= tol and maxerr(dv3, rv) <= tol and bool((dq3 == 7.0).all())
    dk3.fill_(7.0); dv3.fill_(7.0)
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq3, None, None, causal, scale, accumulate=False)
    torch.cuda.synchronize()
    assert maxerr(dq3, rq) <= tol and bool((dk3 == 7.0).all()) and bool((dv3 == 7.0).all())


@pytest.mark.parametrize("shape", SHAPES_F32)
def test_pair_f32(shape):
    _run_pair(torch.float32, *shape)


@pytest.mark.parametrize("shape", SHAPES_BF16)
def test_pair_bf16(shape):
    _run_pair(torch.bfloat16, *shape)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_pair_token_major_layout(dtype, d):
    """Operands laid out [tokens, heads, d] (sequence stride = heads * d, head stride = d) and seen as
    [heads, tokens, d] views: every stride in the shape descriptor differs from the packed case."""
    h_q, h_kv, s_q, s_k, causal = 4, 2, 200, 200, True
    q, k, v, do = case(4242, h_q, h_kv, s_q, s_k, d, dtype)
    scale = 1 / math.sqrt(d)

    def tm(t):        # same values, token-major storage
        return t.permute(1, 0, 2).contiguous().to(dev()).permute(1, 0, 2)

    Q, K, V, dO = tm(q), tm(k), tm(v), tm(do)
    assert Q.stride() == (d, h_q * d, 1)
    o = torch.empty(s_q, h_q, d, device=dev()).permute(1, 0, 2)
    lse = torch.empty(h_q, s_q, device=dev())
    dfa.dfa_chunk_fwd(Q, K, V, causal, scale, o=o, lse=lse)
    delta = dfa.dfa_delta(o, dO)
    dq = torch.zeros(s_q, h_q, d, device=dev()).permute(1, 0, 2)
    dk = torch.zeros(s_k, h_kv, d, device=dev()).permute(1, 0, 2)
    dv = torch.zeros(s_k, h_kv, d, device=dev()).permute(1, 0, 2)
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, causal, scale, accumulate=False)
    torch.cuda.synchronize()
    O, L, rq, rk, rv = _pair_oracle(q, k, v, do, scale, causal)
    tol = TOL[dtype]
    errs = dict(o=maxerr(o, O), lse=maxerr(lse, L), dq=maxerr(dq, rq), dk=maxerr(dk, rk), dv=maxerr(dv, rv))
    assert all(e <= tol for e in errs.values()), errs


def test_pair_bf16_output_dtype_bf16():
    _run_pair(torch.bfloat16, 2, 2, 256, 256, 128, True, o_dtype=torch.bfloat16)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("d", [64, 128])
def test_merge(dtype, d):
    rows_h, rows_s = 3, 1000
    g = torch.Generator().manual_seed(3)
    o_a = torch.randn(rows_h, rows_s, d, generator=g).to(dtype); o_b = torch.randn(rows_h, rows_s, d, generator=g).to(dtype)
    l_a = 3 * torch.randn(rows_h, rows_s, generator=g); l_b = 3 * torch.randn(rows_h, rows_s, generator=g)
    # identities and degenerate rows
    l_a[0, :10] = -math.inf; o_a[0, :10] = 0
    l_b[0, 5:20] = -math.inf; o_b[0, 5:20] = 0
    l_a[1, 0] = 80.0; l_b[1, 0] = -80.0
    want_o, want_l = A.merge(np64(o_a), np64(l_a), np64(o_b), np64(l_b))
    A_, LA = o_a.to(dev()), l_a.to(dev())
    dfa.dfa_merge(A_, LA, o_b.to(dev()), l_b.to(dev()))
    torch.cuda.synchronize()
    got_o, got_l = np64(A_), np64(LA)
    assert not np.isnan(got_o).any() and not np.isnan(got_l).any()
    fin = np.isfinite(want_l)
    assert np.array_equal(np.isneginf(got_l), np.isneginf(want_l))
    assert np.abs(got_l[fin] - want_l[fin]).max() <= 1e-5
    assert np.abs(got_o - want_o).max() <= TOL[dtype]
    assert np.all(got_o[0, 5:10] == 0)


def test_merge_strided_rows():
    d = 128
    big = torch.randn(2, 64, 2 * d).to(dev())
    o_a = big[:, :, :d]          # row stride 2d
    o_b = torch.randn(2, 64, d).to(dev())
    l_a = torch.randn(2, 64).to(dev()); l_b = torch.randn(2, 64).to(dev())
    want_o, want_l = A.merge(np64(o_a), np64(l_a), np64(o_b), np64(l_b))
    keep = big[:, :, d:].clone()
    dfa.dfa_merge(o_a, l_a, o_b, l_b)
    torch.cuda.synchronize()
    assert maxerr(o_a, want_o) <= 1e-5 and maxerr(l_a, want_l) <= 1e-5
    assert torch.equal(big[:, :, d:], keep)      # neighbours untouched


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_empty_key_chunk_gives_merge_identity(dtype):
    d = 128
    q = torch.randn(2, 96, d).to(dtype).to(dev())
    k = torch.empty(2, 0, d, dtype=dtype, device=dev())
    o, lse = dfa.dfa_chunk_fwd(q, k, k, False, 0.1)
    torch.cuda.synchronize()
    assert torch.all(o == 0) and torch.all(torch.isneginf(lse))
    # merging it into a real partial changes nothing
    k2 = torch.randn(2, 64, d).to(dtype).to(dev())
    o2, l2 = dfa.dfa_chunk_fwd(q, k2, k2, False, 0.1)
    ref_o, ref_l = o2.clone(), l2.clone()
    dfa.dfa_merge(o2, l2, o, lse)
    torch.cuda.synchronize()
    assert torch.equal(o2, ref_o) and torch.equal(l2, ref_l)


def _schedule_case(w: dfa_inputs.Workload, mode="balanced", fused=True):
    q, k, v, do = (dfa_inputs.full_sequence(w, t) for t in range(4))
    Q, K, V, dO = (t.to(dev()) for t in (q, k, v, do))
    bufs = driver.Buffers(w.h_q, w.h_kv, w.n_total, w.d, w.p, dev())
    driver.run_all_workers(Q, K, V, dO, w.scale, w.p, bufs, mode=mode, fused=fused)
    torch.cuda.synchronize()
    q64, k64, v64, do64 = (np64(t) for t in (q, k, v, do))
    if isinstance(mode, tuple):     # ("window", W): attention local to the W preceding chunks
        O, L = A.window_attention_fwd(q64, k64, v64, w.scale, w.n_total // w.p, mode[1])
        dQ, dK, dV = A.window_attention_bwd(q64, k64, v64, do64, w.scale, w.n_total // w.p, mode[1])
    else:
        O, L = A.attention_fwd(q64, k64, v64, w.scale)
        dQ, dK, dV = A.attention_bwd(q64, k64, v64, do64, w.scale)
    tol = TOL[w.torch_dtype]
    errs = dict(o=maxerr(bufs.O, O), lse=maxerr(bufs.L, L), dq=maxerr(bufs.dQ, dQ), dk=maxerr(bufs.dK, dK),
                dv=maxerr(bufs.dV, dV))
    assert all(e <= tol for e in errs.values()), errs
    return errs


@pytest.mark.parametrize("fused", [True, False])
def test_config1_full_balanced_schedule(fused):
    """Config 1: fp32, 1 head, d=64, N=1024, P=4; merged outputs of the whole schedule vs the monolithic oracle.
    fused: OWN pairs continue from the owner's state (dfa_chunk_fwd_acc); else partial + dfa_merge."""
    _schedule_case(dfa_inputs.CONFIGS[0], fused=fused)


@pytest.mark.parametrize("fused", [True, False])
def test_config1_ring_schedule(fused):
    _schedule_case(dfa_inputs.CONFIGS[0], mode="ring", fused=fused)


@pytest.mark.parametrize("W", [0, 1, 2, 9])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_window_schedule(W, dtype):
    """Local sliding window at chunk granularity (appendix on sparse patterns): the truncated
    schedule's merged outputs and summed gradients against the oracle's windowed attention."""
    w = dfa_inputs.Workload(f"t_win{W}", 4, 2, 128, 160 * 5, 5, dtype, 777 + W)
    _schedule_case(w, mode=("window", W))
    if W == 1:
        _schedule_case(w, mode=("window", W), fused=False)


@pytest.mark.parametrize("P", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_balanced_schedule_odd_even_gqa(P, dtype):
    w = dfa_inputs.Workload(f"t_p{P}", 4, 2, 128, 192 * P, P, dtype, 4321 + P)
    _schedule_case(w)
    if P in (3, 8):
        _schedule_case(w, fused=False)


@pytest.mark.parametrize("dtype,d,o_dtype", [(torch.float32, 64, torch.float32), (torch.float32, 128, torch.float32),
                                             (torch.bfloat16, 128, torch.float32),
                                             (torch.bfloat16, 128, torch.bfloat16)])
def test_chunk_fwd_acc_chain(dtype, d, o_dtype):
    """attn(q, k_r, v_r, o, s) over three key/value chunks of ragged sizes, started from the empty
    state (lse = -inf over a poisoned o): equals attention over the concatenated keys (oracle), and
    equals partial + merge up to rounding; an empty chunk leaves the state untouched."""
    h_q, h_kv, s_q = 4, 2, 200
    sizes = [200, 77, 130]            # the first chunk is the causal diagonal one
    scale = 1 / math.sqrt(d)
    g = torch.Generator().manual_seed(77)
    q = torch.randn(h_q, s_q, d, generator=g).to(dtype)
    ks = [torch.randn(h_kv, n, d, generator=g).to(dtype) for n in sizes]
    vs = [torch.randn(h_kv, n, d, generator=g).to(dtype) for n in sizes]
    Q = q.to(dev())
    o = torch.full((h_q, s_q, d), float("nan"), dtype=o_dtype, device=dev())
    lse = torch.full((h_q, s_q), -math.inf, device=dev())
    o_m = l_m = None
    for i, (k, v) in enumerate(zip(ks, vs)):
        K, V = k.to(dev()), v.to(dev())
        dfa.dfa_chunk_fwd_acc(Q, K, V, i == 0, scale, o, lse)
        po, pl = dfa.dfa_chunk_fwd(Q, K, V, i == 0, scale, o_dtype=o_dtype)
        if o_m is None:
            o_m, l_m = po, pl
        else:
            dfa.dfa_merge(o_m, l_m, po, pl)
    keep_o, keep_l = o.clone(), lse.clone()
    empty = torch.empty(h_kv, 0, d, dtype=dtype, device=dev())
    dfa.dfa_chunk_fwd_acc(Q, empty, empty, False, scale, o, lse)
    torch.cuda.synchronize()
    assert torch.equal(o, keep_o) and torch.equal(lse, keep_l)
    # oracle: chunk 0 causal, chunks 1 and 2 unmasked, each the monolithic definition over that chunk's
    # keys, combined with the oracle's merge (pinned on the CPU to equal attention over all the keys)
    q64 = np64(q)
    O, L = A.attention_fwd(q64, np64(ks[0]), np64(vs[0]), scale, causal=True)
    for k, v in zip(ks[1:], vs[1:]):
        O, L = A.merge(O, L, *A.attention_fwd(q64, np64(k), np64(v), scale, causal=False))
    tol = TOL[dtype] if o_dtype == torch.float32 else 2e-2
    assert maxerr(o, O) <= tol and maxerr(lse, L) <= (1e-5 if dtype == torch.float32 else 2e-2)
    assert maxerr(o, np64(o_m)) <= (2e-5 if (dtype == torch.float32) else 2e-2)
    # (bf16: the forward sums the bf16-rounded weights, whose rounding differs between the two routes)
    assert maxerr(lse, np64(l_m)) <= (1e-5 if dtype == torch.float32 else 5e-3)


def test_forward_with_staged_kv_equals_direct():
    """OWN pairs reading key/value chunks staged one step ahead on a second stream (the overlap of
    Section 3.2 emulated with a device-to-device copy) match the oracle and are bit-identical to the
    direct path, run after run."""
    w = dfa_inputs.Workload("t_prefetch", 4, 2, 128, 256 * 8, 8, "bf16", 777)
    q, k, v, _ = (dfa_inputs.full_sequence(w, t) for t in range(4))
    Q, K, V = (t.to(dev()) for t in (q, k, v))
    worker = w.p - 1
    ref = driver.Buffers(w.h_q, w.h_kv, w.n_total, w.d, w.p, dev(), grads=False)
    driver.forward_worker(Q, K, V, w.scale, w.p, worker, ref, mode="ring")
    pf = driver.KVPrefetcher(K, V, w.chunk)
    c = w.chunk
    # under the ring schedule worker P-1 computes all its pairs itself: its rows of plain causal attention
    O, L = A.attention_fwd(np64(q), np64(k), np64(v), w.scale)
    assert maxerr(ref.O[:, worker * c:], O[:, worker * c:]) <= TOL[torch.bfloat16]
    assert maxerr(ref.L[:, worker * c:], L[:, worker * c:]) <= TOL[torch.bfloat16]
    for _ in range(3):
        got = driver.Buffers(w.h_q, w.h_kv, w.n_total, w.d, w.p, dev(), grads=False)
        driver.forward_worker(Q, K, V, w.scale, w.p, worker, got, mode="ring", prefetch=pf)
        torch.cuda.synchronize()
        assert maxerr(got.O[:, worker * c:], O[:, worker * c:]) <= TOL[torch.bfloat16]
        assert maxerr(got.L[:, worker * c:], L[:, worker * c:]) <= TOL[torch.bfloat16]
        assert torch.equal(got.O[:, worker * c:], ref.O[:, worker * c:])
        assert torch.equal(got.L[:, worker * c:], ref.L[:, worker * c:])


@pytest.mark.parametrize("causal", [False, True])
def test_forward_running_maximum_moves(causal):
    """Scores that grow along the key axis by far more than the lazy-maximum threshold (2^8 in the
    exp2 domain per step): every tile moves the reference and rescales O and the row sum; the
    backward sees probabilities spanning the whole exponent range."""
    h, s, d = 2, 1024, 128
    g = torch.Generator().manual_seed(5)
    q = torch.randn(h, s, d, generator=g)
    k = torch.randn(h, s, d, generator=g) * 0.3
    # add to every key a component along each query's mean direction, growing with the key index
    u = q.mean(1, keepdim=True); u = u / u.norm(dim=-1, keepdim=True)
    ramp = torch.linspace(0.0, 60.0, s).view(1, s, 1)
    k = k + ramp * u
    q = q + 4.0 * u                      # q.u ~ 4 -> scaled scores ramp up to ~ 60 * 4 / sqrt(128) = 21 (2^30)
    v = torch.randn(h, s, d, generator=g)
    do = torch.randn(h, s, d, generator=g)
    q, k, v, do = (t.to(torch.bfloat16) for t in (q, k, v, do))
    scale = 1 / math.sqrt(d)
    Q, K, V, dO = (t.to(dev()) for t in (q, k, v, do))
    o, lse = dfa.dfa_chunk_fwd(Q, K, V, causal, scale)
    # the same through two halves of the keys with the state carried over
    if not causal:
        o2 = torch.zeros_like(o); l2 = torch.full_like(lse, -math.inf)
        dfa.dfa_chunk_fwd_acc(Q, K[:, :512], V[:, :512], False, scale, o2, l2)
        dfa.dfa_chunk_fwd_acc(Q, K[:, 512:], V[:, 512:], False, scale, o2, l2)
    delta = dfa.dfa_delta(o, dO)
    dq = torch.zeros(h, s, d, device=dev()); dk = torch.zeros_like(dq); dv = torch.zeros_like(dq)
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, causal, scale)
    torch.cuda.synchronize()
    O, L, rq, rk, rv = _pair_oracle(q, k, v, do, scale, causal)
    assert float(L.max() - L.min()) > 12.0          # the logsumexp itself spans many e-folds across rows
    tol = TOL[torch.bfloat16]
    errs = dict(o=maxerr(o, O), lse=maxerr(lse, L), dq=maxerr(dq, rq), dk=maxerr(dk, rk), dv=maxerr(dv, rv))
    if not causal:
        errs.update(o_acc=maxerr(o2, O), lse_acc=maxerr(l2, L))
    # gradients here reach magnitudes of tens: bound them relative to their scale as well
    scale_of = dict(o=1.0, lse=1.0, o_acc=1.0, lse_acc=1.0, dq=max(1.0, np.abs(rq).max()),
                    dk=max(1.0, np.abs(rk).max()), dv=max(1.0, np.abs(rv).max()))
    assert all(errs[n] <= tol * scale_of[n] for n in errs), (errs, scale_of)


@pytest.mark.parametrize("top", [600.0, 6000.0])
def test_forward_reference_jumps(top):
    """Scores that jump by far more per 64-key tile than the forward's stale reference tolerates
    (2^14 in the exp2 domain; with the larger ramp the exponentials against the old reference
    overflow to infinity): every tile has to be redone against a moved reference, and key tiles in
    a random order make the reference both jump and stay.  Full pair and the same from two halves."""
    h, s_q, s_k, d = 2, 300, 1024 + 37, 128
    g = torch.Generator().manual_seed(11)
    q = torch.randn(h, s_q, d, generator=g)
    k = torch.randn(h, s_k, d, generator=g) * 0.3
    u = q.mean(1, keepdim=True); u = u / u.norm(dim=-1, keepdim=True)
    ramp = torch.linspace(0.0, top, s_k)
    # whole 64-key tiles in shuffled order: some tiles tower over everything before them, others lie far below
    order = torch.randperm((s_k + 63) // 64, generator=g)
    ramp = torch.cat([ramp[i * 64:(i + 1) * 64] for i in order.tolist()]).view(1, s_k, 1)
    k = k + ramp * u
    q = q + 4.0 * u
    v = torch.randn(h, s_k, d, generator=g)
    q, k, v = (t.to(torch.bfloat16) for t in (q, k, v))
    scale = 1 / math.sqrt(d)
    Q, K, V = (t.to(dev()) for t in (q, k, v))
    o, lse = dfa.dfa_chunk_fwd(Q, K, V, False, scale)
    o2 = torch.zeros_like(o); l2 = torch.full_like(lse, -math.inf)
    dfa.dfa_chunk_fwd_acc(Q, K[:, :512], V[:, :512], False, scale, o2, l2)
    dfa.dfa_chunk_fwd_acc(Q, K[:, 512:], V[:, 512:], False, scale, o2, l2)
    torch.cuda.synchronize()
    O, L = A.attention_fwd(np64(q), np64(k), np64(v), scale, causal=False)
    assert float(L.max()) > 0.2 * top * 4 * scale          # the logsumexp is as large as the ramp makes it
    tol = TOL[torch.bfloat16]
    # lse is hundreds to thousands here and is formed in fp32 from scores of that size: allow 2^-17 of it
    ltol = max(tol, float(np.abs(L).max()) * 2.0 ** -17)
    errs = dict(o=maxerr(o, O), o_acc=maxerr(o2, O))
    lerrs = dict(lse=maxerr(lse, L), lse_acc=maxerr(l2, L))
    assert all(e <= tol for e in errs.values()) and all(e <= ltol for e in lerrs.values()), (errs, lerrs, ltol)


def test_mfma_probe_runs_and_counts_its_flop():
    out = torch.empty(512 * 256, dtype=torch.float32, device=dev())
    flop = dfa.dfa_mfma_probe(out, 100)
    torch.cuda.synchronize()
    assert flop == 2.0 * 32 * 32 * 16 * 4 * 100 * 2048
    assert bool(torch.isfinite(out).all())


def test_mfma_probe_data_runs_and_counts_its_flop():
    ops = torch.randn(1 << 20, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16).to(dev())
    out = torch.empty(512 * 256, dtype=torch.float32, device=dev())
    flop = dfa.dfa_mfma_probe_data(ops, out, 100)
    torch.cuda.synchronize()
    assert flop == 2.0 * 32 * 32 * 16 * 8 * 100 * 2048
    assert bool(torch.isfinite(out).all())


@pytest.mark.parametrize("shape", [(4, 2, 333, 451, False, 12), (8, 2, 257, 257, True, 12), (32, 8, 1024, 2048, False, 6)])
def test_results_repeat_bit_for_bit(shape):
    """The kernels use no atomics and a fixed summation order, so repeated calls must agree bit for
    bit; a difference would point at a missing wait or barrier between the tile copies, the
    hand-over buffers and their readers (the last shape fills every compute unit)."""
    h_q, h_kv, s_q, s_k, causal, reps = shape
    d = 128
    q, k, v, do = case(4242 + s_q, h_q, h_kv, s_q, s_k, d, torch.bfloat16)
    Q, K, V, dO = (t.to(dev()) for t in (q, k, v, do))
    scale = 1 / math.sqrt(d)
    first = None
    for _ in range(reps):
        o, lse = dfa.dfa_chunk_fwd(Q, K, V, causal, scale)
        delta = dfa.dfa_delta(o, dO)
        dq = torch.empty(h_q, s_q, d, device=dev()); dk = torch.empty(h_kv, s_k, d, device=dev())
        dv = torch.empty(h_kv, s_k, d, device=dev())
        dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, causal, scale, accumulate=False)
        torch.cuda.synchronize()
        cur = (o, lse, delta, dq, dk, dv)
        if first is None:
            first = cur
        else:
            assert all(torch.equal(a, b) for a, b in zip(first, cur))


SENTINEL = 12345.0
RAGGED = sorted({s for s in SHAPES_BF16 + SHAPES_F32 if s[2] % 64 or s[3] % 64})


def _framed(h, s, d, dtype, rows=3, cols=8):
    """A [h, s, d] view in the middle of a larger tensor filled with a sentinel: `rows` rows before
    and after every head's rows, one head before and after, `cols` columns on both sides of d.
    Returns (view, frame, mask of the frame's elements outside the view)."""
    frame = torch.full((h + 2, s + 2 * rows, d + 2 * cols), SENTINEL, dtype=dtype, device=dev())
    view = frame[1:-1, rows:rows + s, cols:cols + d]
    outside = torch.ones_like(frame, dtype=torch.bool)
    outside[1:-1, rows:rows + s, cols:cols + d] = False
    return view, frame, outside


def _framed_rows(h, s, rows=3):
    frame = torch.full((h + 2, s + 2 * rows), SENTINEL, dtype=torch.float32, device=dev())
    view = frame[1:-1, rows:rows + s]
    outside = torch.ones_like(frame, dtype=torch.bool)
    outside[1:-1, rows:rows + s] = False
    return view, frame, outside


@pytest.mark.parametrize("shape", RAGGED, ids=lambda s: "x".join(str(int(x)) for x in s))
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_ragged_outputs_stay_inside_their_slices(shape, dtype):
    """Out-of-bounds guard for ragged chunk lengths: every output (o, lse, D, dq, dk, dv, the merge's
    in-place operand) is an interior slice of a larger tensor filled with a sentinel; after forward,
    forward-from-state, merge, D pre-pass and backward (overwriting, then accumulating) the sentinel
    rows, columns and heads around the slices must be untouched, and the slices must hold the
    oracle's values."""
    h_q, h_kv, s_q, s_k, d, causal = shape
    if dtype == torch.bfloat16 and d != 128:
        pytest.skip("bf16 kernels take d = 128")
    q, k, v, do = case(2000 + s_q + s_k, h_q, h_kv, s_q, s_k, d, dtype)
    scale = 1 / math.sqrt(d)
    Q, K, V, dO = (t.to(dev()) for t in (q, k, v, do))
    frames = []

    def framed(h, s, dt=torch.float32):
        view, frame, outside = _framed(h, s, d, dt)
        frames.append((frame, outside))
        return view

    def framed_rows(h, s):
        view, frame, outside = _framed_rows(h, s)
        frames.append((frame, outside))
        return view

    o, lse = framed(h_q, s_q), framed_rows(h_q, s_q)
    o2, lse2 = framed(h_q, s_q), framed_rows(h_q, s_q)
    o3, lse3 = framed(h_q, s_q), framed_rows(h_q, s_q)
    delta = framed_rows(h_q, s_q)
    dq, dk, dv = framed(h_q, s_q), framed(h_kv, s_k), framed(h_kv, s_k)
    dfa.dfa_chunk_fwd(Q, K, V, causal, scale, o=o, lse=lse)
    # the same pair continued from the empty state (lse = -inf), then merged into a copy of itself
    lse2.fill_(-math.inf)
    dfa.dfa_chunk_fwd_acc(Q, K, V, causal, scale, o2, lse2)
    o3.copy_(o); lse3.copy_(lse)
    dfa.dfa_merge(o3, lse3, o2, lse2)
    dfa.dfa_delta(o, dO, delta=delta)
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, causal, scale, accumulate=False)
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, causal, scale, accumulate=True)
    torch.cuda.synchronize()
    for frame, outside in frames:
        assert bool((frame[outside] == SENTINEL).all()), "a kernel wrote outside its output slice"
    O, L, rq, rk, rv = _pair_oracle(q, k, v, do, scale, causal)
    tol = TOL[dtype]
    errs = dict(o=maxerr(o, O), lse=maxerr(lse, L), o_acc=maxerr(o2, O), lse_acc=maxerr(lse2, L),
                o_merged=maxerr(o3, O), lse_merged=maxerr(lse3, L + math.log(2.0)),
                dq=maxerr(dq, 2 * rq), dk=maxerr(dk, 2 * rk), dv=maxerr(dv, 2 * rv))
    # the gradients here are twice one contribution, and with grouped heads and short causal rows
    # they reach |x| ~ 10, where 1e-5 is a dozen fp32 ulps: bound them relative to their magnitude
    mag = dict(dq=max(1.0, 2 * np.abs(rq).max()), dk=max(1.0, 2 * np.abs(rk).max()), dv=max(1.0, 2 * np.abs(rv).max()))
    assert all(errs[n] <= tol * mag.get(n, 1.0) for n in errs), (errs, mag)
