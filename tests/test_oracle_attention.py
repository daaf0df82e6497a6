"""Pins for oracle/attention.py against things other than itself: finite
differences, PyTorch's CPU softmax / autograd, closed forms and invariants.
Each pin is chosen so that a dropped term, a wrong sign or index or a transposed
operand in the oracle fails at least one of them."""
import math

import numpy as np
import pytest
import torch

import dfa_inputs
from oracle import attention as A


def _np(*ts):
    return [t.to(torch.float64).numpy() for t in ts]


def _case(seed, h_q, h_kv, n, d):
    return _np(*dfa_inputs.small_case(seed, h_q, h_kv, n, d))


# ----------------------------------------------------------------- forward
def test_softmax_rows_sum_to_one_and_causal():
    q, k, v, do = _case(1, 4, 2, 37, 8)
    P = A.softmax_weights(q, k, 0.3)
    assert np.abs(P.sum(-1) - 1).max() < 1e-14
    assert np.all(np.triu(P, 1) == 0)          # no weight on future keys
    assert np.all(np.diagonal(P, axis1=1, axis2=2) > 0)  # a token attends to itself


def test_row0_and_equal_keys_closed_forms():
    q, k, v, do = _case(2, 2, 2, 33, 16)
    scale = 0.25
    O, L = A.attention_fwd(q, k, v, scale)
    # row 0 sees one key: O_0 = V_0, L_0 = scale q0.k0
    assert np.abs(O[:, 0] - v[:, 0]).max() < 1e-14
    assert np.abs(L[:, 0] - scale * (q[:, 0] * k[:, 0]).sum(-1)).max() < 1e-13
    # all keys equal -> uniform weights: O_i = prefix mean of V, L_i = c_i + log(i+1)
    k2 = np.broadcast_to(k[:, :1], k.shape).copy()
    O2, L2 = A.attention_fwd(q, k2, v, scale)
    pref = np.cumsum(v, axis=1) / np.arange(1, 34)[None, :, None]
    assert np.abs(O2 - pref).max() < 1e-13
    c = scale * np.einsum("hnd,hd->hn", q, k[:, 0])
    assert np.abs(L2 - (c + np.log(np.arange(1, 34))[None])).max() < 1e-12
    # V constant along the sequence -> O equals that constant
    v3 = np.broadcast_to(v[:, :1], v.shape).copy()
    O3, _ = A.attention_fwd(q, k, v3, scale)
    assert np.abs(O3 - v3).max() < 1e-13


def test_key_shift_invariance():
    q, k, v, do = _case(3, 2, 1, 29, 8)
    scale = 0.4
    c = np.linspace(-1, 1, 8)
    O, L = A.attention_fwd(q, k, v, scale)
    O2, L2 = A.attention_fwd(q, k + c, v, scale)
    assert np.abs(O - O2).max() < 1e-12
    assert np.abs(L2 - (L + scale * q @ c)).max() < 1e-12


@pytest.mark.parametrize("h_q,h_kv,n,d", [(2, 2, 48, 16), (4, 1, 65, 8), (8, 2, 130, 32)])
def test_forward_matches_torch_softmax(h_q, h_kv, n, d):
    """Special case that is a library routine: masked softmax + matmul in torch fp64."""
    tq, tk, tv, tdo = [t.double() for t in dfa_inputs.small_case(7, h_q, h_kv, n, d)]
    scale = 1 / math.sqrt(d)
    g = h_q // h_kv
    kk = tk.repeat_interleave(g, 0); vv = tv.repeat_interleave(g, 0)
    s = scale * tq @ kk.transpose(1, 2)
    s = s.masked_fill(torch.triu(torch.ones(n, n, dtype=torch.bool), 1), float("-inf"))
    ref_o = torch.softmax(s, -1) @ vv
    ref_l = torch.logsumexp(s, -1)
    O, L = A.attention_fwd(tq.numpy(), tk.numpy(), tv.numpy(), scale, row_block=32)
    assert np.abs(O - ref_o.numpy()).max() < 1e-13
    assert np.abs(L - ref_l.numpy()).max() < 1e-13
    # and torch's fused CPU attention
    sdpa = torch.nn.functional.scaled_dot_product_attention(
        tq[None], kk[None], vv[None], is_causal=True, scale=scale)[0]
    assert np.abs(O - sdpa.numpy()).max() < 1e-12


# ---------------------------------------------------------------- backward
def test_backward_finite_differences():
    q, k, v, do = _case(11, 2, 1, 12, 6)
    scale = 0.37

    def loss(q_, k_, v_):
        return float((A.attention_fwd(q_, k_, v_, scale)[0] * do).sum())

    dq, dk, dv = A.attention_bwd(q, k, v, do, scale)
    eps = 1e-6
    rng = np.random.default_rng(0)
    for arr, grad, idx in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        for _ in range(40):
            pos = tuple(rng.integers(0, s) for s in arr.shape)
            args = [q.copy(), k.copy(), v.copy()]
            args[idx][pos] += eps
            up = loss(*args)
            args[idx][pos] -= 2 * eps
            dn = loss(*args)
            fd = (up - dn) / (2 * eps)
            assert abs(fd - grad[pos]) <= 1e-7 * max(1.0, abs(fd)), (idx, pos, fd, grad[pos])


@pytest.mark.parametrize("h_q,h_kv,n,d", [(2, 2, 40, 16), (4, 2, 67, 8)])
def test_backward_matches_torch_autograd(h_q, h_kv, n, d):
    tq, tk, tv, tdo = [t.double() for t in dfa_inputs.small_case(13, h_q, h_kv, n, d)]
    scale = 1 / math.sqrt(d)
    g = h_q // h_kv
    tq.requires_grad_(True); tk.requires_grad_(True); tv.requires_grad_(True)
    s = scale * tq @ tk.repeat_interleave(g, 0).transpose(1, 2)
    s = s.masked_fill(torch.triu(torch.ones(n, n, dtype=torch.bool), 1), float("-inf"))
    o = torch.softmax(s, -1) @ tv.repeat_interleave(g, 0)
    o.backward(tdo)
    dq, dk, dv = A.attention_bwd(tq.detach().numpy(), tk.detach().numpy(), tv.detach().numpy(),
                                 tdo.numpy(), scale, row_block=16)
    assert np.abs(dq - tq.grad.numpy()).max() < 1e-12
    assert np.abs(dk - tk.grad.numpy()).max() < 1e-12
    assert np.abs(dv - tv.grad.numpy()).max() < 1e-12


def test_backward_invariants():
    q, k, v, do = _case(17, 4, 2, 50, 8)
    scale = 0.3
    dq, dk, dv = A.attention_bwd(q, k, v, do, scale)
    g = 2
    # softmax rows sum to 1  ->  sum_j dV_j = sum_i dO_i over the group's query heads
    assert np.abs(dv.sum(1) - do.reshape(2, g, 50, 8).sum((1, 2))).max() < 1e-12
    # shift invariance in k  ->  sum_j dK_j = 0
    assert np.abs(dk.sum(1)).max() < 1e-12
    # S depends on q.k only  ->  <Q,dQ> = <K,dK>
    assert abs((q * dq).sum() - (k * dk).sum()) < 1e-10
    # row 0 has a single key: its softmax is constant, so dQ_0 = 0
    assert np.abs(dq[:, 0]).max() < 1e-14
    # V constant along the sequence -> O constant -> dQ = dK = 0
    v3 = np.broadcast_to(v[:, :1], v.shape).copy()
    dq3, dk3, _ = A.attention_bwd(q, k, v3, do, scale)
    assert np.abs(dq3).max() < 1e-12 and np.abs(dk3).max() < 1e-12


def test_delta_identity():
    q, k, v, do = _case(19, 2, 2, 30, 8)
    O, _ = A.attention_fwd(q, k, v, 0.5)
    P = A.softmax_weights(q, k, 0.5)
    dP = do @ np.swapaxes(v, 1, 2)
    assert np.abs(A.delta_rows(O, do) - (P * dP).sum(-1)).max() < 1e-13


# ----------------------------------------------- unmasked rectangular pairs (s_q != s_k)
@pytest.mark.parametrize("h_q,h_kv,s_q,s_k,d", [(3, 1, 23, 41, 8), (4, 2, 50, 17, 16), (2, 2, 1, 9, 4)])
def test_unmasked_rectangular_pair_matches_torch(h_q, h_kv, s_q, s_k, d):
    """causal=False with different numbers of query and key rows (a query chunk against an earlier,
    ragged key/value chunk): forward against torch's fp64 softmax / logsumexp, backward against
    torch autograd; grouped heads sum into their key/value head."""
    g = torch.Generator().manual_seed(31 + s_q)
    tq = torch.randn(h_q, s_q, d, generator=g, dtype=torch.float64, requires_grad=True)
    tdo = torch.randn(h_q, s_q, d, generator=g, dtype=torch.float64)
    tk = torch.randn(h_kv, s_k, d, generator=g, dtype=torch.float64, requires_grad=True)
    tv = torch.randn(h_kv, s_k, d, generator=g, dtype=torch.float64, requires_grad=True)
    scale = 0.3
    grp = h_q // h_kv
    s = scale * tq @ tk.repeat_interleave(grp, 0).transpose(1, 2)
    o = torch.softmax(s, -1) @ tv.repeat_interleave(grp, 0)
    o.backward(tdo)
    q, k, v, do = (t.detach().numpy() for t in (tq, tk, tv, tdo))
    O, L = A.attention_fwd(q, k, v, scale, causal=False, row_block=16)
    assert O.shape == (h_q, s_q, d) and L.shape == (h_q, s_q)
    assert np.abs(O - o.detach().numpy()).max() < 1e-13
    assert np.abs(L - torch.logsumexp(s, -1).detach().numpy()).max() < 1e-13
    dq, dk, dv = A.attention_bwd(q, k, v, do, scale, causal=False, row_block=16)
    assert dk.shape == k.shape and dv.shape == v.shape
    assert np.abs(dq - tq.grad.numpy()).max() < 1e-12
    assert np.abs(dk - tk.grad.numpy()).max() < 1e-12
    assert np.abs(dv - tv.grad.numpy()).max() < 1e-12


def test_causal_chunk_then_unmasked_ragged_chunks_merge_to_softmax_over_all_keys():
    """A causal square chunk followed by unmasked chunks of other sizes, merged: equals torch's
    softmax over the concatenated keys under the combined mask."""
    h_q, h_kv, s_q, d, scale = 4, 2, 13, 8, 0.4
    sizes = [13, 5, 21]
    g = torch.Generator().manual_seed(5)
    tq = torch.randn(h_q, s_q, d, generator=g, dtype=torch.float64)
    ks = [torch.randn(h_kv, n, d, generator=g, dtype=torch.float64) for n in sizes]
    vs = [torch.randn(h_kv, n, d, generator=g, dtype=torch.float64) for n in sizes]
    O, L = A.attention_fwd(tq.numpy(), ks[0].numpy(), vs[0].numpy(), scale, causal=True)
    for k, v in zip(ks[1:], vs[1:]):
        O, L = A.merge(O, L, *A.attention_fwd(tq.numpy(), k.numpy(), v.numpy(), scale, causal=False))
    kk = torch.cat(ks, 1).repeat_interleave(2, 0); vv = torch.cat(vs, 1).repeat_interleave(2, 0)
    s = scale * tq @ kk.transpose(1, 2)
    mask = torch.zeros(s_q, sum(sizes), dtype=torch.bool)
    mask[:, :sizes[0]] = torch.triu(torch.ones(s_q, sizes[0], dtype=torch.bool), 1)
    s = s.masked_fill(mask, float("-inf"))
    assert np.abs(O - (torch.softmax(s, -1) @ vv).numpy()).max() < 1e-13
    assert np.abs(L - torch.logsumexp(s, -1).numpy()).max() < 1e-13


# ------------------------------------------------- chunk pairs and merging
@pytest.mark.parametrize("P", range(1, 10))
def test_merged_pair_partials_equal_monolithic(P):
    c, d = 6, 8
    q, k, v, do = _case(100 + P, 4, 2, P * c, d)
    scale = 1 / math.sqrt(d)
    O, L = A.attention_fwd(q, k, v, scale)
    D = A.delta_rows(O, do)
    dQ, dK, dV = A.attention_bwd(q, k, v, do, scale)
    aq = np.zeros_like(dQ); ak = np.zeros_like(dK); av = np.zeros_like(dV)
    for p in range(P):
        o_acc = np.zeros((4, c, d)); l_acc = np.full((4, c), -np.inf)
        order = list(range(p + 1))
        if P % 2:
            order.reverse()            # merge order must not matter
        for r in order:
            o_p, l_p = A.pair_fwd(q, k, v, scale, p, r, c)
            o_acc, l_acc = A.merge(o_acc, l_acc, o_p, l_p)
            dq, dk, dv = A.pair_bwd(q, k, v, do, L, D, scale, p, r, c)
            aq[:, p * c:(p + 1) * c] += dq
            ak[:, r * c:(r + 1) * c] += dk
            av[:, r * c:(r + 1) * c] += dv
        assert np.abs(o_acc - O[:, p * c:(p + 1) * c]).max() < 1e-12
        assert np.abs(l_acc - L[:, p * c:(p + 1) * c]).max() < 1e-12
    assert np.abs(aq - dQ).max() < 1e-12
    assert np.abs(ak - dK).max() < 1e-12
    assert np.abs(av - dV).max() < 1e-12


def test_merge_identity_commutative_and_two_key_closed_form():
    rng = np.random.default_rng(5)
    o_a = rng.normal(size=(3, 7, 4)); o_b = rng.normal(size=(3, 7, 4))
    l_a = rng.normal(size=(3, 7)); l_b = rng.normal(size=(3, 7))
    o0 = np.zeros_like(o_a); l0 = np.full_like(l_a, -np.inf)
    o, l = A.merge(o0, l0, o_a, l_a)
    assert np.array_equal(o, o_a) and np.array_equal(l, l_a)
    o, l = A.merge(o_a, l_a, o0, l0)
    assert np.array_equal(o, o_a) and np.array_equal(l, l_a)
    o, l = A.merge(o0, l0, o0, l0)
    assert not np.isnan(o).any() and np.all(np.isneginf(l))
    o1, l1 = A.merge(o_a, l_a, o_b, l_b)
    o2, l2 = A.merge(o_b, l_b, o_a, l_a)
    assert np.abs(o1 - o2).max() < 1e-15 and np.abs(l1 - l2).max() < 1e-15
    # closed form: weights are the two-way softmax of (l_a, l_b)
    wa = 1 / (1 + np.exp(l_b - l_a))
    assert np.abs(o1 - (wa[..., None] * o_a + (1 - wa)[..., None] * o_b)).max() < 1e-14
    assert np.abs(l1 - np.log(np.exp(l_a) + np.exp(l_b))).max() < 1e-14


def test_row_and_column_samplers_match_full():
    c, P, d = 8, 4, 8
    q, k, v, do = _case(23, 4, 2, P * c, d)
    scale = 0.35
    O, L = A.attention_fwd(q, k, v, scale)
    D = A.delta_rows(O, do)
    dQ, dK, dV = A.attention_bwd(q, k, v, do, scale)
    rows = np.array([0, 7, 8, 19, 31])
    h, kh = 3, 1
    o_r, l_r = A.rows_fwd(q[h, rows], rows, k[kh], v[kh], scale)
    assert np.abs(o_r - O[h, rows]).max() < 1e-13 and np.abs(l_r - L[h, rows]).max() < 1e-13
    dq_r = A.rows_dq(q[h, rows], rows, do[h, rows], L[h, rows], D[h, rows], k[kh], v[kh], scale)
    assert np.abs(dq_r - dQ[h, rows]).max() < 1e-13
    cols = np.array([0, 5, 16, 31])
    dk_c = np.zeros((4, d)); dv_c = np.zeros((4, d))
    for hh in (2, 3):
        a, b = A.cols_dkdv(k[kh, cols], v[kh, cols], cols, q[hh], do[hh], L[hh], D[hh], scale)
        dk_c += a; dv_c += b
    assert np.abs(dk_c - dK[kh, cols]).max() < 1e-13 and np.abs(dv_c - dV[kh, cols]).max() < 1e-13


# ----------------------------------------------------------------- chunk-level local window
def test_window_brute_force_and_limits():
    """The windowed attention against pure-Python loops over the kept keys, its two limits
    (window >= P-1: plain causal attention; window 0: every chunk on its own) and the
    worked example of the appendix (window of one worker: worker 7 sees workers 6 and 7)."""
    h_q, h_kv, c, P, d = 2, 1, 5, 4, 3
    n = c * P
    q, k, v, do = _case(41, h_q, h_kv, n, d)
    scale = 0.41
    for w in (0, 1, 2):
        O, L = A.window_attention_fwd(q, k, v, scale, c, w)
        for h in range(h_q):
            for i in range(n):
                keys = [j for j in range(i + 1) if j // c >= i // c - w]
                z = [math.exp(scale * sum(q[h, i, x] * k[0, j, x] for x in range(d))) for j in keys]
                tot = sum(z)
                for x in range(d):
                    ref = sum(zj * v[0, j, x] for zj, j in zip(z, keys)) / tot
                    assert abs(O[h, i, x] - ref) < 1e-12
                assert abs(L[h, i] - math.log(tot)) < 1e-12
    Of, Lf = A.attention_fwd(q, k, v, scale)
    Ow, Lw = A.window_attention_fwd(q, k, v, scale, c, P - 1)
    assert np.abs(Of - Ow).max() < 1e-14 and np.abs(Lf - Lw).max() < 1e-14
    O0, L0 = A.window_attention_fwd(q, k, v, scale, c, 0)
    for p in range(P):
        sl = slice(p * c, (p + 1) * c)
        Oc, Lc = A.attention_fwd(q[:, sl], k[:, sl], v[:, sl], scale)
        assert np.abs(O0[:, sl] - Oc).max() < 1e-14 and np.abs(L0[:, sl] - Lc).max() < 1e-14
    # P = 8, window of one worker: the last worker's rows depend on chunks 6 and 7 only
    c8 = 3
    q8, k8, v8, _ = _case(43, 1, 1, 8 * c8, 4)
    O1, _ = A.window_attention_fwd(q8, k8, v8, 0.5, c8, 1)
    k8b, v8b = k8.copy(), v8.copy()
    k8b[:, :6 * c8] += 3.0; v8b[:, :6 * c8] -= 2.0
    O2, _ = A.window_attention_fwd(q8, k8b, v8b, 0.5, c8, 1)
    assert np.array_equal(O1[:, 7 * c8:], O2[:, 7 * c8:])
    assert not np.allclose(O1[:, 6 * c8:7 * c8], O2[:, 6 * c8:7 * c8])   # worker 6 does see chunk 5


def test_window_backward_finite_differences_and_merge_of_pairs():
    h_q, h_kv, c, P, d = 2, 1, 4, 3, 5
    n = c * P
    q, k, v, do = _case(47, h_q, h_kv, n, d)
    scale, w = 0.37, 1

    def loss(q_, k_, v_):
        return float((A.window_attention_fwd(q_, k_, v_, scale, c, w)[0] * do).sum())

    dq, dk, dv = A.window_attention_bwd(q, k, v, do, scale, c, w)
    eps = 1e-6
    rng = np.random.default_rng(1)
    for arr, grad, idx in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        for _ in range(40):
            pos = tuple(rng.integers(0, s) for s in arr.shape)
            args = [q.copy(), k.copy(), v.copy()]
            args[idx][pos] += eps
            up = loss(*args)
            args[idx][pos] -= 2 * eps
            dn = loss(*args)
            fd = (up - dn) / (2 * eps)
            assert abs(fd - grad[pos]) <= 1e-7 * max(1.0, abs(fd)), (idx, pos, fd, grad[pos])
    # the truncated schedule's pairs, merged, give the windowed attention; their backward
    # contributions, summed, its gradients
    O, L = A.window_attention_fwd(q, k, v, scale, c, w)
    D = A.delta_rows(O, do)
    gq, gk, gv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for p in range(P):
        o_p, l_p = A.pair_fwd(q, k, v, scale, p, p, c)
        for r in range(max(0, p - w), p):
            o_p, l_p = A.merge(o_p, l_p, *A.pair_fwd(q, k, v, scale, p, r, c))
        assert np.abs(o_p - O[:, p * c:(p + 1) * c]).max() < 1e-13
        assert np.abs(l_p - L[:, p * c:(p + 1) * c]).max() < 1e-13
        for r in range(max(0, p - w), p + 1):
            a, b, e = A.pair_bwd(q, k, v, do, L, D, scale, p, r, c)
            gq[:, p * c:(p + 1) * c] += a; gk[:, r * c:(r + 1) * c] += b; gv[:, r * c:(r + 1) * c] += e
    assert np.abs(gq - dq).max() < 1e-12 and np.abs(gk - dk).max() < 1e-12 and np.abs(gv - dv).max() < 1e-12
