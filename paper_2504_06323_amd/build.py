"""Compile the HIP kernels and the C-ABI into csrc/libmosaic_prune.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB_PATH = os.path.join(CSRC, "libmosaic_prune.so")
SOURCES = ["stats.hip", "score.hip", "rank_batch.hip", "select.hip", "structured.hip", "groups.hip", "plan_device.hip", "hessian.hip", "factor.hip", "sweep.hip", "mlp.hip", "layer.hip", "attention.hip", "host.cpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                   # the metric multiply must never fuse into a sum
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-Wno-unknown-warning-option",
]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", INCLUDE, "-I", CSRC]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += ["-x", "hip", path]
    cmd += ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, cwd=CSRC, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature and says so once per kernel: not an error
    noise = "'-packed-fp32-ops' is not a recognized feature for this target"
    out = "\n".join(l for l in proc.stdout.splitlines() if noise not in l)
    if out.strip() and (verbose or proc.returncode):
        print(out, flush=True)
    if proc.returncode:
        raise RuntimeError(f"hipcc failed with exit code {proc.returncode}")
    return LIB_PATH


if __name__ == "__main__":
    build()
    sys.exit(0)
