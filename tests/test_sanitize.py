"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the CPU-side code (no GPU):
the fp64 oracle, driven on small inputs of every storage type, and the host side
of the C ABI (argument checks, planning arithmetic, workspace sizes), driven over
a sweep of shapes up to INT_MAX with the kernel launchers stubbed out.  Both
drivers live in tests/sanitize/; a sanitizer report makes the run exit non-zero.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
# (another preloaded library may precede the sanitizer runtime in the library list: that order is not checked)
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, " ".join(cmd) + "\n" + p.stdout[-4000:]
    return p.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", *SAN, "-fopenmp", "-std=c11", "-ffp-contract=off", "-o", exe,
          os.path.join(ROOT, "tests", "sanitize", "oracle_san_main.c"), os.path.join(ROOT, "oracle", "fdd_oracle.c"), "-lm"])
    out = _run([exe], env=dict(ENV, OMP_NUM_THREADS="4"))
    assert "oracle sanitizer run: ok" in out


def test_abi_host_code_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "abi_san")
    host = []
    for f in SAN:                  # host pass only: the device pass has no sanitizer support on this target
        host += ["-Xarch_host", f]
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
          "-I" + os.path.join(ROOT, "paper_2605_23163_amd", "csrc"), *host, "-Wno-unused-command-line-argument",
          "-Wno-option-ignored", "-x", "hip", os.path.join(ROOT, "paper_2605_23163_amd", "csrc", "api.hip"),
          "-x", "hip", os.path.join(ROOT, "tests", "sanitize", "abi_host_san_main.cpp"), "-fsanitize=address,undefined",
          "-o", exe])
    out = _run([exe], env=ENV)
    assert "ABI host sanitizer run: ok" in out
