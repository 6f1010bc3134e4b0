"""Host-side hardening (no GPU): the C oracle and the host half of the C-ABI library built with the address and
undefined-behaviour sanitizers and driven over their argument space (tests/host/*).  The drivers exit non-zero on
a failed expectation; the sanitizers abort with a report on any bad access, overflow or misaligned use.
The sanitized binaries live under _build/ (not the product build) and are rebuilt when a source is newer."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "_build", "host_asan")
CSRC = os.path.join(ROOT, "paper_2507_05753_amd", "csrc")


def stale(target, sources):
    return not os.path.exists(target) or any(os.path.getmtime(s) > os.path.getmtime(target) for s in sources)


def run(binary):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([binary], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_under_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_driver")
    src = [os.path.join(ROOT, "oracle", "jigsaw_oracle.c"), os.path.join(ROOT, "tests", "host", "oracle_driver.c")]
    if stale(exe, src):
        subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-fsanitize=address,undefined",
                               "-static-libasan", "-fno-omit-frame-pointer", "-pthread", *src, "-o", exe, "-lm"])
    assert "0 failures" in run(exe)


@pytest.mark.timeout(900)
def test_c_abi_host_half_under_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "abi_driver")
    src = [os.path.join(CSRC, "jigsaw.hip"), os.path.join(ROOT, "tests", "host", "abi_driver.cpp")]
    deps = src + [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "jigsaw.h")]
    if stale(exe, deps):
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        # the sanitizers instrument the host pass only (each flag right behind -Xarch_host); the device pass is the
        # product's, at a low optimisation level to keep the build short
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
                               "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                               "-Xarch_host", "-fno-omit-frame-pointer",
                               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *src, "-o", exe],
                              stderr=subprocess.DEVNULL)
    out = run(exe)
    assert "0 failures" in out and "plans exercised" in out
