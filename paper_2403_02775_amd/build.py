"""Builds libeasyquant.so (the C-ABI library) for gfx950 with hipcc, in-tree.

The host side and the small kernels are one translation unit; each family of lane kernels is a
translation unit of its own, compiled once per input type, and all of them are compiled side by
side (objects go to _build/, which is not part of the repository)."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libeasyquant.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # the arithmetic contract: no fused multiply-add is formed
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # atomics are issued by single lanes here; the compiler's wave-level rewrite of them would
    # wait for the returned value at once instead of where it is used
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-fvisibility=hidden", "-Wall", "-Wno-unused-command-line-argument",
]

# (source file, EQ_TU_DT or None): EQ_TU_DT is the input type a family unit is instantiated for
UNITS = [("easyquant_api.hip", None)] + [(f, dt) for f in ("eq_tu_units.hip", "eq_tu_channels.hip", "eq_tu_rtn.hip", "eq_tu_sorted.hip")
                                         for dt in (0, 1)]


def sources():
    return [os.path.join(CSRC, f) for f in sorted({f for f, _ in UNITS})]


def build(verbose: bool = False, jobs: int = 8) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    os.makedirs(OBJ_DIR, exist_ok=True)
    common = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    pending = []
    for src, dt in UNITS:
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ("" if dt is None else f"_dt{dt}") + ".o")
        cmd = [*common, "-c", os.path.join(CSRC, src), "-o", obj] + ([] if dt is None else [f"-DEQ_TU_DT={dt}"])
        pending.append((cmd, obj))
    objs, running = [], []
    for cmd, obj in pending:
        if verbose:
            print(" ".join(cmd), flush=True)
        running.append((subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True), cmd))
        objs.append(obj)
        if len(running) >= jobs:
            _finish(running.pop(0), verbose)
    for r in running:
        _finish(r, verbose)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", "-o", LIB, *objs]
    if verbose:
        print(" ".join(link), flush=True)
    res = subprocess.run(link, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc (link) failed:\n" + res.stdout + res.stderr)
    return LIB


def _finish(job, verbose):
    proc, cmd = job
    out, _ = proc.communicate()
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
    if verbose and out.strip():
        print(out)


if __name__ == "__main__":
    print(build(verbose=True))
