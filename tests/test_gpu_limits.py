"""GPU parity at the edges of what the ABI accepts: the longest key/value chunk the 32-bit offsets allow
(rows * sequence stride * 4 < 2^31, i.e. 4194303 rows at d = 128) and a large number of heads."""
import math

import numpy as np
import pytest
import torch

import paper_2310_03294_amd as dfa
from oracle import attention as A
from gpu_util import TOL, dev, maxerr, np64

pytestmark = pytest.mark.gpu


def test_longest_key_chunk():
    """One head, 32 query rows against 4194303 keys, the most the limit admits (ragged: the last tile
    holds 63 rows): the last dk / dv rows end 512 bytes below the 2^31-byte offset."""
    d, s_q = 128, 32
    scale = 1 / math.sqrt(d)
    g = torch.Generator().manual_seed(17)
    for s_k in (4194303,):
        q = torch.randn(1, s_q, d, generator=g).to(torch.bfloat16)
        do = torch.randn(1, s_q, d, generator=g).to(torch.bfloat16)
        k = torch.randn(1, s_k, d, generator=g).to(torch.bfloat16)
        v = torch.randn(1, s_k, d, generator=g).to(torch.bfloat16)
        Q, K, V, dO = (t.to(dev()) for t in (q, k, v, do))
        o, lse = dfa.dfa_chunk_fwd(Q, K, V, False, scale)
        delta = dfa.dfa_delta(o, dO)
        dq = torch.empty(1, s_q, d, device=dev())
        dk = torch.empty(1, s_k, d, device=dev()); dv = torch.empty(1, s_k, d, device=dev())
        dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, False, scale)
        torch.cuda.synchronize()
        O, L = A.attention_fwd(np64(q), np64(k), np64(v), scale, causal=False)
        rq, rk, rv = A.attention_bwd(np64(q), np64(k), np64(v), np64(do), scale, causal=False)
        tol = TOL[torch.bfloat16]
        errs = dict(o=maxerr(o, O), lse=maxerr(lse, L), dq=maxerr(dq, rq))
        # dk, dv in slabs, to bound the fp64 copies; the tail slab is the one next to the offset limit
        for name, got, want in (("dk", dk, rk), ("dv", dv, rv)):
            e = 0.0
            for r0 in range(0, s_k, 1 << 20):
                e = max(e, maxerr(got[:, r0:r0 + (1 << 20)], want[:, r0:r0 + (1 << 20)]))
            errs[name] = e
            errs[name + "_tail"] = maxerr(got[:, -256:], want[:, -256:])
        assert all(x <= tol for x in errs.values()), (s_k, errs)
        # one row more is refused before anything is launched
        if s_k == 4194303:
            kk = torch.empty(1, s_k + 1, d, dtype=torch.bfloat16, device=dev())
            with pytest.raises(dfa.DfaError):
                dfa.dfa_chunk_bwd(Q, kk, kk, lse, delta, dO, dq, torch.empty(1, s_k + 1, d, device=dev()),
                                  torch.empty(1, s_k + 1, d, device=dev()), False, scale)
        del K, V, dk, dv, rk, rv
        torch.cuda.empty_cache()


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_many_heads(dtype, d):
    """8192 query heads in groups of 4 (grid sizes and head offsets far beyond the Llama shapes)."""
    h_q, h_kv, s = 8192, 2048, 96
    scale = 1 / math.sqrt(d)
    g = torch.Generator().manual_seed(23)
    q = torch.randn(h_q, s, d, generator=g).to(dtype); do = torch.randn(h_q, s, d, generator=g).to(dtype)
    k = torch.randn(h_kv, s, d, generator=g).to(dtype); v = torch.randn(h_kv, s, d, generator=g).to(dtype)
    Q, K, V, dO = (t.to(dev()) for t in (q, k, v, do))
    o, lse = dfa.dfa_chunk_fwd(Q, K, V, True, scale)
    delta = dfa.dfa_delta(o, dO)
    dq = torch.empty(h_q, s, d, device=dev()); dk = torch.empty(h_kv, s, d, device=dev()); dv = torch.empty_like(dk)
    dfa.dfa_chunk_bwd(Q, K, V, lse, delta, dO, dq, dk, dv, True, scale)
    torch.cuda.synchronize()
    O, L = A.attention_fwd(np64(q), np64(k), np64(v), scale)
    rq, rk, rv = A.attention_bwd(np64(q), np64(k), np64(v), np64(do), scale)
    tol = TOL[dtype]
    errs = dict(o=maxerr(o, O), lse=maxerr(lse, L), dq=maxerr(dq, rq), dk=maxerr(dk, rk), dv=maxerr(dv, rv))
    # grouped heads and short causal rows: gradients reach |x| ~ 10, bound them relative to their magnitude
    mag = dict(dq=max(1.0, np.abs(rq).max()), dk=max(1.0, np.abs(rk).max()), dv=max(1.0, np.abs(rv).max()))
    assert all(errs[n] <= tol * mag.get(n, 1.0) for n in errs), (errs, mag)
