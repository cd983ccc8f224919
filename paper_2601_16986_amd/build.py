"""Builds libckv.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libckv.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-ffp-contract=off",                       # CRF update and Alg. 2 must round as written
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep the fused kernel's queue atomic a plain atomic: the wave-level rewrite of atomics reads the
    # result back at once, and that wait is a wait for every load in flight
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the ckv library cannot be built")


def build_library(verbose: bool = False) -> str:
    """Compile csrc/ckv.hip into libckv.so; always recompiles."""
    cmd = [hipcc_path(), *HIPCC_FLAGS, os.path.join(CSRC, "ckv.hip"), "-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
