"""Build the C-ABI library ``libcg_conv.so`` from ``csrc/`` with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
LIB = PKG / "libcg_conv.so"

SOURCES = ["cg_conv_api.hip", "kernels_naive.hip", "kernels_mfma3.hip", "kernels_dense.hip",
           "kernels_tile.hip", "kernels_tile_bf16_k3.hip", "kernels_tile_bf16_k1.hip", "kernels_tile_i8_k3.hip",
           "kernels_tile_i8_k1.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
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


def build(verbose: bool = False, extra=(), jobs: int = 6) -> Path:
    """Compile every source every time it is called (the 'does it build' check): one object per
    source, compiled side by side, then one link."""
    cc = hipcc()
    work = Path(tempfile.mkdtemp(prefix="cg_build_"))
    try:
        def compile_one(src: str) -> str:
            obj = work / (src + ".o")
            cmd = [cc, *FLAGS, *extra, "-I", str(ROOT / "include"), "-I", str(CSRC), "-c", str(CSRC / src),
                   "-o", str(obj)]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
            return str(obj)

        with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        tmp = LIB.with_name(LIB.name + ".tmp%d" % os.getpid())
        link = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", str(tmp)]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.check_call(link)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
