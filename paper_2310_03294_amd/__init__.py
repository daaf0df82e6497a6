"""MI355X-native DistFlashAttn per-worker hot path: thin Python binding over libdfa.so.

Every step of the path runs in the HIP kernels of the C-ABI library; this package only
marshals arguments (device pointers, sizes, strides, the current HIP stream).  There is
no CPU or PyTorch fallback: if the library has not been built, loading fails loudly.
"""
from .binding import (  # noqa: F401
    DfaError,
    Step,
    dfa_chunk_bwd,
    dfa_chunk_fwd,
    dfa_chunk_fwd_acc,
    dfa_delta,
    dfa_merge,
    dfa_mfma_probe,
    dfa_mfma_probe_data,
    dfa_schedule,
    dfa_status_str,
    dfa_version,
    lib_path,
    load_library,
)
from .driver import run_worker_share, run_all_workers  # noqa: F401
