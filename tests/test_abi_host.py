"""CPU-only checks of the C-ABI library: it loads, exports every function the header
declares, validates arguments on the host (no launch on error), and its schedule equals
the oracle's enumerator."""
import ctypes
import os
import re

import pytest

import paper_2310_03294_amd as dfa
from paper_2310_03294_amd import binding as B
from oracle import schedule as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dfa.lib_path()):
        import __graft_entry__ as g
        g.build()
    return dfa.load_library()


def test_exports_every_declared_symbol(lib):
    hdr = open(os.path.join(ROOT, "include", "dfa.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(dfa_[a-z_]+)\s*\(", hdr))
    assert {"dfa_chunk_fwd", "dfa_merge", "dfa_chunk_bwd", "dfa_schedule", "dfa_delta"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert set(B.EXPORTS) == names
    assert lib.dfa_version() >= 100


def test_shape_struct_matches_header():
    # 10 32-bit fields then 11 64-bit strides
    assert ctypes.sizeof(B.DfaShape) == 10 * 4 + 11 * 8
    assert ctypes.sizeof(B.DfaStep) == 24


@pytest.mark.parametrize("P", list(range(1, 34)) + [64])
def test_schedule_matches_oracle(lib, P):
    for mode, ref in (("balanced", S.balanced(P)), ("ring", S.ring(P))):
        for w in range(P):
            got = dfa.dfa_schedule(P, w, mode)
            want = ref[w]
            assert len(got) == len(want)
            for g, r in zip(got, want):
                assert g._asdict() == r


@pytest.mark.parametrize("P", [1, 2, 5, 8, 16])
def test_window_schedule_matches_oracle(lib, P):
    for W in (0, 1, 3, P - 1, P + 4):
        ref = S.window(P, W)
        for w in range(P):
            got = dfa.dfa_schedule(P, w, ("window", W))
            assert [g._asdict() for g in got] == ref[w]
    buf = (B.DfaStep * 2)()
    assert lib.dfa_schedule_window(P, 0, -1, buf, 2) == -4
    assert lib.dfa_schedule_window(P, P, 1, buf, 2) == -4
    assert lib.dfa_schedule_window(P, 0, 1, None, 2) == -1


def test_mfma_probe_rejects_bad_arguments_before_any_launch(lib):
    flop = ctypes.c_double(0)
    assert lib.dfa_mfma_probe(None, 1 << 20, 10, ctypes.byref(flop), None) == -1
    assert lib.dfa_mfma_probe(ctypes.c_void_p(256), 1 << 20, 0, ctypes.byref(flop), None) == -4
    assert lib.dfa_mfma_probe(ctypes.c_void_p(256), 1000, 10, ctypes.byref(flop), None) == -4


def test_mfma_probe_data_rejects_bad_arguments_before_any_launch(lib):
    flop = ctypes.c_double(0)
    ok = ctypes.c_void_p(4096)
    assert lib.dfa_mfma_probe_data(None, 1 << 20, ok, 1 << 20, 10, ctypes.byref(flop), None) == -1
    assert lib.dfa_mfma_probe_data(ok, 1 << 20, None, 1 << 20, 10, ctypes.byref(flop), None) == -1
    assert lib.dfa_mfma_probe_data(ok, (1 << 20) - 16, ok, 1 << 20, 10, ctypes.byref(flop), None) == -4
    assert lib.dfa_mfma_probe_data(ok, 1 << 20, ok, 1 << 20, 0, ctypes.byref(flop), None) == -4
    assert lib.dfa_mfma_probe_data(ok, 1 << 20, ok, 1000, 10, ctypes.byref(flop), None) == -4
    assert lib.dfa_mfma_probe_data(ctypes.c_void_p(4100), 1 << 20, ok, 1 << 20, 10, ctypes.byref(flop), None) == -2


def test_schedule_errors_and_cap(lib):
    buf = (B.DfaStep * 2)()
    assert lib.dfa_schedule(0, 0, buf, 2) == -4
    assert lib.dfa_schedule(4, 4, buf, 2) == -4
    assert lib.dfa_schedule(4, -1, buf, 2) == -4
    assert lib.dfa_schedule(4, 0, None, 2) == -1
    assert lib.dfa_schedule(8, 7, buf, 2) == 5          # truncated write, full count returned
    assert buf[1].kind == B.DFA_STEP_OWN and buf[1].kv_chunk == 6 and buf[1].recv_from == 0
    assert lib.dfa_schedule(8, 7, None, 0) == 5
    assert lib.dfa_schedule_mode(7, 8, 0, buf, 2) == -4


def _shape(**kw):
    sh = B.DfaShape()
    base = dict(h_q=2, h_kv=2, s_q=64, s_k=64, d=64, dtype=B.DFA_F32, o_dtype=B.DFA_F32, causal=0, scale=0.125,
                reserved=0, q_stride_h=64 * 64, q_stride_s=64, kv_stride_h=64 * 64, kv_stride_s=64,
                o_stride_h=64 * 64, o_stride_s=64, lse_stride_h=64, dq_stride_h=64 * 64, dq_stride_s=64,
                dkv_stride_h=64 * 64, dkv_stride_s=64)
    base.update(kw)
    for k, v in base.items():
        setattr(sh, k, v)
    return sh


FAKE = 4096  # non-null, 16-byte aligned, never dereferenced: validation fails before any launch


@pytest.mark.parametrize("kw,code", [
    (dict(d=96), -2), (dict(h_q=3, h_kv=2), -2), (dict(s_q=-1), -2), (dict(dtype=5), -3), (dict(o_dtype=9), -3),
    (dict(causal=1, s_k=128), -4), (dict(causal=2), -4), (dict(scale=0.0), -4), (dict(scale=float("nan")), -4),
    (dict(reserved=1), -4), (dict(q_stride_s=60), -2), (dict(kv_stride_s=63), -2), (dict(o_stride_h=12), -2),
    (dict(lse_stride_h=32), -2), (dict(dtype=B.DFA_BF16, d=64), -2),
    # one head's slice of a chunk is addressed with 32-bit byte offsets: rows * row stride * 4 < 2^31
    (dict(s_q=1 << 20, lse_stride_h=1 << 20, q_stride_s=512, q_stride_h=1 << 29), -2),
    (dict(s_k=1 << 21, kv_stride_s=256, kv_stride_h=1 << 29), -2),
])
def test_fwd_argument_errors(lib, kw, code):
    sh = _shape(**kw)
    assert lib.dfa_chunk_fwd(ctypes.byref(sh), FAKE, FAKE, FAKE, FAKE, FAKE, None) == code
    assert code < 0 and dfa.dfa_status_str(code) != "unknown dfa_status"


def test_null_and_alignment_errors(lib):
    sh = _shape()
    assert lib.dfa_chunk_fwd(None, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -1
    assert lib.dfa_chunk_fwd(ctypes.byref(sh), None, FAKE, FAKE, FAKE, FAKE, None) == -1
    assert lib.dfa_chunk_fwd(ctypes.byref(sh), FAKE + 4, FAKE, FAKE, FAKE, FAKE, None) == -2
    assert lib.dfa_chunk_bwd(ctypes.byref(sh), FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, 0, None) == -1
    # outputs: dq alone or (dk, dv) alone are allowed, anything else NULL is not
    assert lib.dfa_chunk_bwd(ctypes.byref(sh), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, 0, None) == -1
    assert lib.dfa_chunk_bwd(ctypes.byref(sh), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 0, None) == -1
    assert lib.dfa_chunk_bwd(ctypes.byref(sh), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None) == -1
    assert lib.dfa_chunk_bwd(ctypes.byref(_shape(dq_stride_s=8)), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                             FAKE, 0, None) == -2
    assert lib.dfa_delta(ctypes.byref(sh), FAKE, None, FAKE, None) == -1
    def md(**kw):
        m = B.DfaMergeDesc()
        base = dict(heads=2, rows=8, d=64, o_dtype=B.DFA_F32, a_stride_h=512, a_stride_s=64, lse_a_stride_h=8,
                    b_stride_h=512, b_stride_s=64, lse_b_stride_h=8)
        base.update(kw)
        for k, v in base.items():
            setattr(m, k, v)
        return ctypes.byref(m)
    assert lib.dfa_merge(md(rows=-1), FAKE, FAKE, FAKE * 2, FAKE * 2, None) == -2
    assert lib.dfa_merge(md(d=48), FAKE, FAKE, FAKE * 2, FAKE * 2, None) == -2
    assert lib.dfa_merge(md(o_dtype=7), FAKE, FAKE, FAKE * 2, FAKE * 2, None) == -3
    assert lib.dfa_merge(md(a_stride_s=60), FAKE, FAKE, FAKE * 2, FAKE * 2, None) == -2
    assert lib.dfa_merge(md(lse_b_stride_h=4), FAKE, FAKE, FAKE * 2, FAKE * 2, None) == -2
    assert lib.dfa_merge(md(), FAKE, FAKE, FAKE, FAKE * 2, None) == -4   # aliasing
    assert lib.dfa_merge(md(), None, FAKE, FAKE * 2, FAKE * 2, None) == -1
    assert lib.dfa_merge(None, FAKE, FAKE, FAKE * 2, FAKE * 2, None) == -1
    assert lib.dfa_merge(md(rows=0, lse_a_stride_h=0, lse_b_stride_h=0), FAKE, FAKE, FAKE * 2, FAKE * 2, None) == 0


def test_empty_query_chunk_is_noop(lib):
    sh = _shape(s_q=0, lse_stride_h=0)
    assert lib.dfa_chunk_fwd(ctypes.byref(sh), FAKE, FAKE, FAKE, FAKE, FAKE, None) == 0
    assert lib.dfa_delta(ctypes.byref(sh), FAKE, FAKE, FAKE, None) == 0
