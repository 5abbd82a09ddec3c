"""Sanitizer builds of the CPU-side code (no GPU): the oracle under AddressSanitizer and
UndefinedBehaviorSanitizer, and the translation unit that validates descriptors and lays out
the caller's buffers, with the host pass of hipcc instrumented the same way."""
import os
import shutil
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SAN = ROOT / "tests" / "sanitize"
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("gcc not found")
    exe = tmp_path / "oracle_driver"
    r = _run(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fopenmp",
              "-Wall", "-o", str(exe), str(SAN / "oracle_driver.c"), "-lm"])
    if r.returncode != 0 and ("asan" in r.stderr.lower() or "ubsan" in r.stderr.lower()) and "cannot find" in r.stderr:
        pytest.skip("sanitizer runtimes are not installed: " + r.stderr[-300:])
    assert r.returncode == 0, r.stderr[-3000:]
    # (the harness's own preloaded library must come after the sanitizer runtime: the driver is a plain
    # executable, so the instrumented runtime is linked in and no preload of ours is needed)
    r = _run([str(exe)], env=dict(ENV, OMP_NUM_THREADS="2", ASAN_OPTIONS=ENV["ASAN_OPTIONS"] + ":verify_asan_link_order=0"))
    assert r.returncode == 0 and "oracle sanitizer driver: ok" in r.stdout, (r.stdout[-2000:], r.stderr[-3000:])


def test_descriptor_validation_under_sanitizers(tmp_path):
    lib = ROOT / "paper_1805_12549_amd" / "libcg_conv.so"
    hipcc = "/opt/rocm/bin/hipcc" if Path("/opt/rocm/bin/hipcc").exists() else shutil.which("hipcc")
    if hipcc is None or not lib.exists():
        pytest.skip("needs hipcc and the built library")
    exe = tmp_path / "abi_driver"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    r = _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *san,
              "-I", str(ROOT / "include"), "-I", str(ROOT / "paper_1805_12549_amd" / "csrc"),
              str(ROOT / "paper_1805_12549_amd" / "csrc" / "cg_conv_api.hip"), str(SAN / "abi_driver.cpp"),
              "-L", str(lib.parent), "-lcg_conv", "-Wl,-rpath," + str(lib.parent), "-o", str(exe)])
    if r.returncode != 0 and "cannot find" in r.stderr and "san" in r.stderr.lower():
        pytest.skip("sanitizer runtimes are not installed: " + r.stderr[-300:])
    assert r.returncode == 0, r.stderr[-3000:]
    r = _run([str(exe)], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:protect_shadow_gap=0"))
    assert r.returncode == 0 and "abi sanitizer driver: ok" in r.stdout, (r.stdout[-2000:], r.stderr[-3000:])
