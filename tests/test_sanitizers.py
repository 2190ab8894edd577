"""CPU builds under -fsanitize=address,undefined: the oracle's C source with a driver that calls every entry point,
and the library's host code (argument checks and host helpers: everything that returns before the first HIP call)
with a driver of its own.  Device code cannot be instrumented here; the kernels' bounds are checked on the GPU by
the guard regions of the parity tests."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, **kw)


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    p = _run(["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off",
              "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan",
              "-o", exe, os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "sidco_oracle.c"), "-lm"])
    assert p.returncode == 0, p.stderr
    r = _run([exe], env=ENV)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "0 failures" in r.stdout and "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stdout + r.stderr


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_library_host_paths_under_address_and_undefined_sanitizers(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    csrc = os.path.join(ROOT, "paper_2101_10761_amd", "csrc")
    exe = str(tmp_path / "api_san")
    srcs = [os.path.join(csrc, s) for s in ("sidco_kernels.hip", "sidco_topk.hip", "sidco_dgc.hip", "sidco_api.hip")]
    cmd = [hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"), "-I", csrc, "-x", "hip", *srcs,
           "-x", "c++", os.path.join(SAN, "api_driver.cpp"), "-fsanitize=address", "-fsanitize=undefined", "-o", exe]
    p = _run(cmd)
    assert p.returncode == 0, "\n".join(l for l in p.stderr.splitlines() if "packed-fp32-ops" not in l)
    r = _run([exe], env=ENV)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "0 failures" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stdout + r.stderr
