"""Build libpbd.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libpbd.so")
SOURCES = [os.path.join(HERE, "csrc", "pbd.hip")]
HEADERS = [os.path.join(HERE, "csrc", "ew_kernels.h"), os.path.join(HERE, "csrc", "conv_kernels.h"),
           os.path.join(HERE, "csrc", "conv_dma_kernels.h"),
           os.path.join(ROOT, "include", "pbd.h")]


def build_lib(verbose: bool = False) -> str:
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # keep MFMA accumulators in ordinary VGPRs: without this the register allocator parks
           # them in AGPRs and copies all of them in and out around the MFMAs of every K step
           "-mllvm", "-amdgpu-mfma-vgpr-form",
           "-I" + os.path.join(ROOT, "include"), *SOURCES, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build_lib(verbose=True))
