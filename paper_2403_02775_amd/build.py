"""Builds libeasyquant.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libeasyquant.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # the arithmetic contract: no fused multiply-add is formed
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # atomics are issued by single lanes here; the compiler's wave-level rewrite of them would
    # wait for the returned value at once instead of where it is used
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-fvisibility=hidden", "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return [os.path.join(CSRC, "easyquant_api.hip")]


def build(verbose: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose and res.stderr.strip():
        print(res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
