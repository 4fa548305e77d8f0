"""Compiles the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import json
import os
import re
import shutil
import subprocess
import tempfile

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


SCAN_REPORT = os.path.join(LIB_DIR, "libpcgrl.scan.json")
_SHIFT64 = re.compile(r"\s*(v_lshlrev_b64|v_lshrrev_b64|v_ashrrev_i64)\s+v\[\d+:\d+\],\s*(\S+),")


def scan_shift_amounts(asm_text: str):
    """Looks through the device assembly of this library for 64-bit vector shifts whose shift
    amount sits in the highest vector register of the kernel's allocation (registers are handed
    out in blocks of eight).  On the MI355X boxes this library is measured on such a shift gives
    wrong results in about a tenth of the lanes once several wavefronts share a SIMD (found with
    the 64x64 maze kernel for wide windows, confirmed with a twenty-line probe kernel: the same
    shift with its amount four registers lower is always right).  The compiler works round this
    for another GPU generation only, so the build checks for it.
    Returns (number of kernels, [(kernel, allocation, instruction), ...])."""
    body, alloc, cur, kern = {}, {}, None, None
    for line in asm_text.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            cur = m.group(1)
            body[cur] = []
            continue
        m = re.match(r"\s*\.amdhsa_kernel (\w+)", line)
        if m:
            kern = m.group(1)
            continue
        m = re.match(r"\s*\.amdhsa_next_free_vgpr (\d+)", line)
        if m and kern:
            alloc[kern] = int(m.group(1))
            continue
        if cur:
            body[cur].append(line)
    found = []
    for k, n in alloc.items():
        top = (n + 7) // 8 * 8 - 1
        for line in body.get(k, []):
            m = _SHIFT64.match(line)
            if m and m.group(2) == f"v{top}":
                found.append((k, top + 1, line.strip()))
    return len(alloc), found


def build(force: bool = True, verbose: bool = False) -> str:
    """Runs hipcc; with force=False only when the library is missing or older than its sources.
    The device assembly the compiler leaves behind is checked by scan_shift_amounts(); a finding
    fails the build (the kernel it names then needs one more register block, see step_kernel)."""
    if force or is_stale():
        os.makedirs(LIB_DIR, exist_ok=True)
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        tmp = tempfile.mkdtemp(prefix="pcgrl_build_")
        try:
            out = os.path.join(tmp, "libpcgrl.so")
            cmd = [hipcc] + HIPCC_FLAGS + ["-save-temps", "-o", out, SRC]
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, cwd=tmp, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            if res.returncode != 0:
                raise RuntimeError("hipcc failed:\n" + res.stdout)
            asm = [f for f in os.listdir(tmp) if f.endswith("gfx950.s")]
            if len(asm) != 1:
                raise RuntimeError("device assembly not found among the compiler's temporaries: %s" % os.listdir(tmp))
            with open(os.path.join(tmp, asm[0])) as f:
                n_kernels, found = scan_shift_amounts(f.read())
            with open(SCAN_REPORT, "w") as f:
                json.dump({"kernels": n_kernels, "findings": found}, f)
            if found:
                raise RuntimeError("64-bit shifts with their amount in the highest allocated vector register:\n" +
                                   "\n".join("  %s (allocation %d): %s" % t for t in found))
            shutil.move(out, LIB)
        finally:
            shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
