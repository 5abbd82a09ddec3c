"""Build the C-ABI library ``libcg_conv.so`` from ``csrc/`` with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
LIB = PKG / "libcg_conv.so"

SOURCES = ["cg_conv_api.hip", "kernels_naive.hip", "kernels_mfma.hip", "kernels_mfma2.hip", "kernels_mfma3.hip", "kernels_dense.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # accumulators stay in ordinary vector registers: with the AGPR form the compiler copies them
    # back and forth around the branches inside the MFMA loops and mis-counts the wait states
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, extra=()) -> Path:
    """Compile every source every time it is called (the 'does it build' check)."""
    tmp = LIB.with_name(LIB.name + ".tmp%d" % os.getpid())
    cmd = [hipcc(), *FLAGS, *extra, "-I", str(ROOT / "include"), "-I", str(CSRC),
           *[str(CSRC / s) for s in SOURCES], "-o", str(tmp)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
