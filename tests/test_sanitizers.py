"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU code: the whole oracle (plain C) and the host
side of the C ABI (the helpers that read host arrays, the workspace and plan queries).  Each is a small program
under tests/sanitize/ that calls the functions on heap blocks of exactly the needed size and exits non-zero, or
prints a sanitizer report, if anything is touched out of bounds.  GPU code is not sanitized (not available here)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    r = _run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-fopenmp",
              os.path.join(ROOT, "oracle", "ss_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-lm", "-o", exe])
    assert r.returncode == 0, r.stdout
    r = _run([exe], env=dict(ENV, OMP_NUM_THREADS="2"), timeout=120)
    assert r.returncode == 0 and "oracle driver done" in r.stdout and "ERROR" not in r.stdout and "runtime error" not in r.stdout, r.stdout


def test_host_side_of_the_abi_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "host_driver")
    csrc = os.path.join(ROOT, "paper_2402_11131_amd", "csrc")
    # the sanitizers go to the host pass only; the device pass is compiled as always
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
           "-fsanitize=undefined", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(csrc, "ss_api.hip"), os.path.join(csrc, "ss_msa.hip"), os.path.join(csrc, "ss_msa_bf16.hip"),
           os.path.join(csrc, "ss_lm_head.hip"), os.path.join(csrc, "ss_tree.hip"), os.path.join(SAN, "host_driver.cpp"),
           "-o", exe]
    r = _run(cmd, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    r = _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"), timeout=120)
    assert r.returncode == 0 and "host driver done" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout
