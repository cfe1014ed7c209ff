"""Host-side sanitizer passes (no GPU): the CPU oracle and the host code of the C ABI layer are built with
AddressSanitizer + UndefinedBehaviorSanitizer and driven through every function / entry point.

* oracle/sanitize_check.c + oracle/fp8_oracle.c -> one executable (gcc, ASan linked statically), every buffer a
  heap block of exactly the documented size;
* tests/abi_sanitize_check.hip + api.hip + tuning.hip -> one executable (hipcc, sanitizers on the host pass only),
  kernel launchers stubbed, so argument validation and workspace planning run for real without a device.
"""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    return r.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "sanitize_check")
        _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
              "-fno-sanitize-recover=all", "-static-libasan", "-o", exe,
              os.path.join(ROOT, "oracle", "sanitize_check.c"), os.path.join(ROOT, "oracle", "fp8_oracle.c"), "-lm"])
        out = _run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1", "OMP_NUM_THREADS": "4"})
        assert "sanitize_check ok" in out


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_abi_host_layer_under_sanitizers_with_stubbed_launchers():
    csrc = os.path.join(ROOT, "paper_2507_16099_amd", "csrc")
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "abi_sanitize_check")
        _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
              "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
              "-Xarch_host", "-fno-sanitize-recover=all",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
              "-o", exe, os.path.join(ROOT, "tests", "abi_sanitize_check.hip"),
              os.path.join(csrc, "api.hip"), os.path.join(csrc, "tuning.hip")])
        # the HIP runtime keeps process-lifetime allocations: leak checking off, everything else on
        out = _run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0"})
        assert "abi_sanitize_check ok" in out
