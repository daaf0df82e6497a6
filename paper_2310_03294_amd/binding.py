"""ctypes binding of include/dfa.h.  Argument marshalling only."""
from __future__ import annotations

import collections
import ctypes
import os

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG_DIR, "libdfa.so")
_lib = None

DFA_BF16, DFA_F32 = 0, 1
DFA_STEP_IDLE, DFA_STEP_DIAG, DFA_STEP_OWN, DFA_STEP_HELP = 0, 1, 2, 3
STEP_NAMES = {0: "idle", 1: "diag", 2: "own", 3: "help"}


class DfaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {dfa_status_str(status)} ({status})")


class DfaShape(ctypes.Structure):
    _fields_ = [
        ("h_q", ctypes.c_int32), ("h_kv", ctypes.c_int32),
        ("s_q", ctypes.c_int32), ("s_k", ctypes.c_int32),
        ("d", ctypes.c_int32), ("dtype", ctypes.c_int32), ("o_dtype", ctypes.c_int32),
        ("causal", ctypes.c_int32), ("scale", ctypes.c_float), ("reserved", ctypes.c_int32),
        ("q_stride_h", ctypes.c_int64), ("q_stride_s", ctypes.c_int64),
        ("kv_stride_h", ctypes.c_int64), ("kv_stride_s", ctypes.c_int64),
        ("o_stride_h", ctypes.c_int64), ("o_stride_s", ctypes.c_int64),
        ("lse_stride_h", ctypes.c_int64),
        ("dq_stride_h", ctypes.c_int64), ("dq_stride_s", ctypes.c_int64),
        ("dkv_stride_h", ctypes.c_int64), ("dkv_stride_s", ctypes.c_int64),
    ]


class DfaMergeDesc(ctypes.Structure):
    _fields_ = [("heads", ctypes.c_int32), ("rows", ctypes.c_int32), ("d", ctypes.c_int32),
                ("o_dtype", ctypes.c_int32),
                ("a_stride_h", ctypes.c_int64), ("a_stride_s", ctypes.c_int64), ("lse_a_stride_h", ctypes.c_int64),
                ("b_stride_h", ctypes.c_int64), ("b_stride_s", ctypes.c_int64), ("lse_b_stride_h", ctypes.c_int64)]


class DfaStep(ctypes.Structure):
    _fields_ = [("t", ctypes.c_int32), ("kind", ctypes.c_int32), ("q_chunk", ctypes.c_int32),
                ("kv_chunk", ctypes.c_int32), ("send_to", ctypes.c_int32), ("recv_from", ctypes.c_int32)]


Step = collections.namedtuple("Step", "t kind q_chunk kv_chunk send_to recv_from")

EXPORTS = ("dfa_chunk_fwd", "dfa_chunk_fwd_acc", "dfa_merge", "dfa_delta", "dfa_chunk_bwd", "dfa_schedule",
           "dfa_schedule_mode", "dfa_schedule_window", "dfa_mfma_probe", "dfa_mfma_probe_data", "dfa_status_str",
           "dfa_version")


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libdfa.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build the HIP extension first "
            "(python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    shp = ctypes.POINTER(DfaShape)
    lib.dfa_chunk_fwd.argtypes = [shp, vp, vp, vp, vp, vp, vp]
    lib.dfa_chunk_fwd_acc.argtypes = [shp, vp, vp, vp, vp, vp, vp]
    lib.dfa_merge.argtypes = [ctypes.POINTER(DfaMergeDesc), vp, vp, vp, vp, vp]
    lib.dfa_delta.argtypes = [shp, vp, vp, vp, vp]
    lib.dfa_chunk_bwd.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp]
    lib.dfa_schedule.argtypes = [i32, i32, ctypes.POINTER(DfaStep), i32]
    lib.dfa_schedule_mode.argtypes = [i32, i32, i32, ctypes.POINTER(DfaStep), i32]
    lib.dfa_schedule_window.argtypes = [i32, i32, i32, ctypes.POINTER(DfaStep), i32]
    lib.dfa_mfma_probe.argtypes = [ctypes.c_void_p, ctypes.c_int64, i32, ctypes.POINTER(ctypes.c_double),
                                   ctypes.c_void_p]
    lib.dfa_mfma_probe_data.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, i32,
                                        ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    lib.dfa_status_str.argtypes = [ctypes.c_int]
    lib.dfa_status_str.restype = ctypes.c_char_p
    lib.dfa_version.argtypes = []
    for name in EXPORTS:
        if name not in ("dfa_status_str",):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def dfa_status_str(status: int) -> str:
    return load_library().dfa_status_str(int(status)).decode()


def dfa_version() -> int:
    return load_library().dfa_version()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return DFA_BF16
    if t.dtype == torch.float32:
        return DFA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _hsd(t: torch.Tensor, name: str):
    if t.dim() != 3 or t.stride(2) != 1:
        raise ValueError(f"{name} must be [heads, seq, d] with unit innermost stride")
    return t.stride(0), t.stride(1)


def _make_shape(q, k, causal, scale, in_dtype, o=None, o_dtype=DFA_F32, lse=None, dq=None, dkv=None) -> DfaShape:
    sh = DfaShape()
    sh.h_q, sh.s_q, sh.d = q.shape
    sh.h_kv, sh.s_k = k.shape[0], k.shape[1]
    sh.dtype, sh.o_dtype = in_dtype, o_dtype
    sh.causal, sh.scale, sh.reserved = int(bool(causal)), float(scale), 0
    sh.q_stride_h, sh.q_stride_s = _hsd(q, "q")
    sh.kv_stride_h, sh.kv_stride_s = _hsd(k, "k")
    if o is not None:
        sh.o_stride_h, sh.o_stride_s = _hsd(o, "o")
    else:
        sh.o_stride_h, sh.o_stride_s = sh.s_q * sh.d, sh.d
    sh.lse_stride_h = lse.stride(0) if lse is not None else sh.s_q
    if dq is not None:
        sh.dq_stride_h, sh.dq_stride_s = _hsd(dq, "dq")
    else:
        sh.dq_stride_h, sh.dq_stride_s = sh.s_q * sh.d, sh.d
    if dkv is not None:
        sh.dkv_stride_h, sh.dkv_stride_s = _hsd(dkv, "dk")
    else:
        sh.dkv_stride_h, sh.dkv_stride_s = sh.s_k * sh.d, sh.d
    return sh


def _check(rc: int, where: str):
    if rc != 0:
        raise DfaError(rc, where)


def dfa_chunk_fwd(q, k, v, causal, scale, o=None, lse=None, o_dtype=torch.float32, stream=None):
    """attn(q_p, k_r, v_r) of one chunk pair from the empty state -> (o, lse)."""
    lib = load_library()
    if v.shape != k.shape or v.stride() != k.stride():
        raise ValueError("k and v must share shape and strides")
    if o is None:
        o = torch.empty(q.shape, dtype=o_dtype, device=q.device)
    if lse is None:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    if lse.stride(1) != 1:
        raise ValueError("lse must have unit innermost stride")
    sh = _make_shape(q, k, causal, scale, _dt(q), o=o, o_dtype=_dt(o), lse=lse)
    _check(lib.dfa_chunk_fwd(ctypes.byref(sh), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                             o.data_ptr(), lse.data_ptr(), _stream(stream)), "dfa_chunk_fwd")
    return o, lse


def dfa_chunk_fwd_acc(q, k, v, causal, scale, o, lse, stream=None):
    """attn(q_p, k_r, v_r, o, s): continues from the state in (o, lse), updates both in place."""
    lib = load_library()
    if v.shape != k.shape or v.stride() != k.stride():
        raise ValueError("k and v must share shape and strides")
    if lse.stride(1) != 1:
        raise ValueError("lse must have unit innermost stride")
    sh = _make_shape(q, k, causal, scale, _dt(q), o=o, o_dtype=_dt(o), lse=lse)
    _check(lib.dfa_chunk_fwd_acc(ctypes.byref(sh), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                 o.data_ptr(), lse.data_ptr(), _stream(stream)), "dfa_chunk_fwd_acc")
    return o, lse


def dfa_merge(o_a, lse_a, o_b, lse_b, stream=None):
    """In place: (o_a, lse_a) <- merge((o_a, lse_a), (o_b, lse_b)).  Tensors [heads, seq, d] / [heads, seq]."""
    lib = load_library()
    if o_a.shape != o_b.shape or lse_a.shape != lse_b.shape or o_a.dtype != o_b.dtype:
        raise ValueError("merge operands must match")
    md = DfaMergeDesc()
    md.heads, md.rows, md.d = o_a.shape
    md.o_dtype = _dt(o_a)
    md.a_stride_h, md.a_stride_s = _hsd(o_a, "o_a")
    md.b_stride_h, md.b_stride_s = _hsd(o_b, "o_b")
    if lse_a.stride(1) != 1 or lse_b.stride(1) != 1:
        raise ValueError("lse must have unit innermost stride")
    md.lse_a_stride_h, md.lse_b_stride_h = lse_a.stride(0), lse_b.stride(0)
    _check(lib.dfa_merge(ctypes.byref(md), o_a.data_ptr(), lse_a.data_ptr(), o_b.data_ptr(), lse_b.data_ptr(),
                         _stream(stream)), "dfa_merge")


def dfa_delta(o, dO, delta=None, stream=None):
    """D = rowsum(dO * O) from the final merged output."""
    lib = load_library()
    if delta is None:
        delta = torch.empty(o.shape[:2], dtype=torch.float32, device=o.device)
    sh = _make_shape(dO, dO, 0, 1.0, _dt(dO), o=o, o_dtype=_dt(o), lse=delta)
    _check(lib.dfa_delta(ctypes.byref(sh), o.data_ptr(), dO.data_ptr(), delta.data_ptr(), _stream(stream)),
           "dfa_delta")
    return delta


def dfa_chunk_bwd(q, k, v, lse, delta, dO, dq, dk, dv, causal, scale, accumulate=False, stream=None):
    """dq, dk, dv contributions of one chunk pair from the saved logsumexp and D (no forward re-run).
    dq=None computes only dk, dv; dk=dv=None computes only dq."""
    lib = load_library()
    if v.shape != k.shape or v.stride() != k.stride():
        raise ValueError("k and v must share shape and strides")
    if dO.shape != q.shape or dO.stride() != q.stride():
        raise ValueError("dO and q must share shape and strides")
    if (dk is None) != (dv is None):
        raise ValueError("dk and dv are given together or not at all")
    if dq is None and dk is None:
        raise ValueError("nothing to compute: dq, dk, dv are all None")
    if dk is not None and (dv.shape != dk.shape or dv.stride() != dk.stride()):
        raise ValueError("dk and dv must share shape and strides")
    if lse.stride() != delta.stride():
        raise ValueError("lse and delta must share strides")
    for t in (dq, dk, dv, lse, delta):
        if t is not None and t.dtype != torch.float32:
            raise TypeError("dq, dk, dv, lse, delta are fp32")
    sh = _make_shape(q, k, causal, scale, _dt(q), lse=lse, dq=dq, dkv=dk)

    def ptr(t):
        return None if t is None else t.data_ptr()

    _check(lib.dfa_chunk_bwd(ctypes.byref(sh), q.data_ptr(), k.data_ptr(), v.data_ptr(), lse.data_ptr(),
                             delta.data_ptr(), dO.data_ptr(), ptr(dq), ptr(dk), ptr(dv),
                             int(bool(accumulate)), _stream(stream)), "dfa_chunk_bwd")
    return dq, dk, dv


def dfa_mfma_probe(out, iters: int, stream=None) -> float:
    """Launches the register-resident MFMA stream (measurement aid); returns its FLOP count."""
    lib = load_library()
    flop = ctypes.c_double(0.0)
    _check(lib.dfa_mfma_probe(out.data_ptr(), out.numel(), int(iters), ctypes.byref(flop), _stream(stream)),
           "dfa_mfma_probe")
    return flop.value


def dfa_mfma_probe_data(operands, out, iters: int, stream=None) -> float:
    """The MFMA stream fed with the values of `operands` (a contiguous bf16 device tensor of at least
    1 MiB); returns its FLOP count."""
    lib = load_library()
    if operands.dtype != torch.bfloat16 or not operands.is_contiguous():
        raise TypeError("operands must be a contiguous bf16 tensor")
    flop = ctypes.c_double(0.0)
    _check(lib.dfa_mfma_probe_data(operands.data_ptr(), operands.numel() * 2, out.data_ptr(), out.numel(),
                                   int(iters), ctypes.byref(flop), _stream(stream)), "dfa_mfma_probe_data")
    return flop.value


def dfa_schedule(P: int, worker_id: int, mode="balanced"):
    """Step list of one worker (host integers only).  mode: "balanced", "ring", or
    ("window", window_chunks) for the local sliding window (dfa_schedule_window)."""
    lib = load_library()
    cap = max(1, P + 1)
    buf = (DfaStep * cap)()
    if isinstance(mode, tuple):
        if mode[0] != "window":
            raise ValueError(mode)
        n = lib.dfa_schedule_window(P, worker_id, int(mode[1]), buf, cap)
    else:
        n = lib.dfa_schedule_mode({"balanced": 0, "ring": 1}[mode], P, worker_id, buf, cap)
    if n < 0:
        raise DfaError(n, "dfa_schedule")
    return [Step(b.t, b.kind, b.q_chunk, b.kv_chunk, b.send_to, b.recv_from) for b in buf[:n]]
