"""First calls from several host threads at once (fresh process, one HIP stream per thread): the
one-time opt-in for large dynamic LDS is taken under std::call_once, so every thread's launches must
succeed and give the single-threaded results bit for bit."""
import os
import subprocess
import sys
import textwrap

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SCRIPT = textwrap.dedent("""
    import sys, threading
    sys.path.insert(0, %r)
    import torch
    import paper_2310_03294_amd as dfa
    dev = torch.device("cuda:0")
    torch.cuda.init()
    h, s_q, s_k, d = 4, 640, 1152, 128
    g = torch.Generator().manual_seed(3)
    q, k, v, do = (torch.randn(h, n, d, generator=g).to(torch.bfloat16).to(dev) for n in (s_q, s_k, s_k, s_q))
    torch.cuda.synchronize()
    results = [None] * 4
    errors = []
    start = threading.Barrier(4)

    def work(i):
        try:
            st = torch.cuda.Stream()
            start.wait()
            with torch.cuda.stream(st):
                o, lse = dfa.dfa_chunk_fwd(q, k, v, False, d ** -0.5)          # first call of the process
                o2, lse2 = dfa.dfa_chunk_fwd(q, k[:, :s_q], v[:, :s_q], True, d ** -0.5)
                delta = dfa.dfa_delta(o, do)
                dq = torch.empty(h, s_q, d, device=dev); dk = torch.empty(h, s_k, d, device=dev); dv = torch.empty_like(dk)
                dfa.dfa_chunk_bwd(q, k, v, lse, delta, do, dq, dk, dv, False, d ** -0.5)
            st.synchronize()
            results[i] = (o, lse, o2, lse2, dq, dk, dv)
        except Exception as e:      # noqa: BLE001
            errors.append(repr(e))

    ts = [threading.Thread(target=work, args=(i,)) for i in range(4)]
    [t.start() for t in ts]; [t.join() for t in ts]
    assert not errors, errors
    for r in results[1:]:
        assert all(torch.equal(a, b) for a, b in zip(results[0], r))
    assert all(bool(torch.isfinite(t).all()) for t in results[0])
    print("threads ok")
""") % ROOT


def test_first_calls_from_four_threads():
    r = subprocess.run([sys.executable, "-c", SCRIPT], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "threads ok" in r.stdout, (r.stdout[-2000:], r.stderr[-3000:])
