"""AddressSanitizer + UndefinedBehaviorSanitizer over the code that runs on the host: the C oracle,
and the library's host logic (plan building, validation, planner).  Each is compiled INTO a small
driver program with the sanitizers on (host code only; no GPU code is instrumented or run) and the
program must finish with status 0 and without a sanitizer report."""
import os
import shutil
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SAN = ROOT / "tests" / "sanitize"
OUT = SAN / "_build"
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, f"{' '.join(map(str, cmd))}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr and "LeakSanitizer" not in r.stderr, r.stderr[-6000:]
    return r.stdout


def test_oracle_under_asan_ubsan():
    OUT.mkdir(exist_ok=True)
    exe = OUT / "driver_oracle"
    _run(["gcc", "-O1", "-g", "-std=c11", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-static-libasan",
          "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-o", str(exe), str(SAN / "driver_oracle.c"),
          str(ROOT / "oracle" / "flexsp_oracle.c"), "-lm"])
    assert "ok" in _run([str(exe)])


def test_host_logic_under_asan_ubsan():
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else shutil.which("hipcc")
    if not hipcc:
        pytest.skip("hipcc not found")
    OUT.mkdir(exist_ok=True)
    exe = OUT / "driver_host"
    csrc = ROOT / "paper_2412_01523_amd" / "csrc"
    # .hip sources as plain C++ for the host (-x c++ would lose <hip/hip_runtime.h>'s host path): hipcc with
    # the sanitizers given to the host compilation only; the files hold no kernels
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-fno-gpu-rdc",
          f"-I{ROOT / 'include'}", f"-I{csrc}", "-o", str(exe), str(SAN / "driver_host.cpp"),
          str(csrc / "flexsp_host.hip"), str(csrc / "planner.hip"), "-fsanitize=address", "-fsanitize=undefined"])
    assert "ok" in _run([str(exe)])
