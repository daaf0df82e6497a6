"""Host code of the library under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

hipcc instruments the HOST pass alone (-Xarch_host), the device code is compiled as usual.  The
driver program calls the pure host functions (schedules) with heap buffers of exactly the size they
may write, and every validating entry point with extreme sizes and strides and never-dereferenced
pointers, so no kernel is launched and no GPU is needed."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2310_03294_amd", "csrc")


def test_host_code_under_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    from paper_2310_03294_amd import build as B
    exe = str(tmp_path / "host_sanitizer_driver")
    srcs = []
    for s in B.SOURCES:
        srcs += (["-x", "hip"] if s.endswith(".cpp") else []) + [os.path.join(CSRC, s)]
    cmd = [hipcc, *B.HIP_FLAGS, "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-g",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, *srcs,
           "-x", "hip", os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "host sanitizer driver: ok" in r.stdout
