"""Compiles the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "pcgrl_api.hip")
DEPS = [SRC, os.path.join(HERE, "csrc", "pcgrl_kernels.hip.h"),
        os.path.join(os.path.dirname(HERE), "include", "pcgrl.h")]
LIB_DIR = os.path.join(HERE, "_lib")
LIB = os.path.join(LIB_DIR, "libpcgrl.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep hipcc from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the reward is a sum of float32 products in a fixed order: no fused multiply-adds
    "-ffp-contract=off",
    # leading scalar kernel arguments (up to 8 of them, 14 dwords) are preloaded into scalar
    # registers at wavefront launch; the step kernel is written for that
    "-mllvm", "-amdgpu-kernarg-preload-count=8",
]


def is_stale() -> bool:
    return (not os.path.exists(LIB)) or os.path.getmtime(LIB) < max(os.path.getmtime(d) for d in DEPS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Runs hipcc; with force=False only when the library is missing or older than its sources."""
    if force or is_stale():
        os.makedirs(LIB_DIR, exist_ok=True)
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB, SRC]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
