"""Compile the HIP kernels and the C-ABI into csrc/libmosaic_prune.so (gfx950 only), and the generator of the
synthetic inputs into csrc/libmosaic_synth.so (a library of its own: it is no part of the pruning path).

Every source is compiled to an object of its own (in parallel, the objects go to csrc/_build/),
then the objects are linked into the shared libraries.  Nothing is cached: every call compiles.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB_PATH = os.path.join(CSRC, "libmosaic_prune.so")
SYNTH_LIB_PATH = os.path.join(CSRC, "libmosaic_synth.so")
OBJ_DIR = os.path.join(CSRC, "_build")
SOURCES = ["stats.hip", "score.hip", "rank_batch.hip", "select.hip", "structured.hip", "groups.hip",
           "plan_device.hip", "hessian.hip", "factor.hip", "sweep.hip", "mlp.hip", "layer.hip", "attention.hip",
           "noalloc.hip", "probe.hip", "host.cpp"]
SYNTH_SOURCES = ["synth_gen.hip"]     # -ffp-contract=off matters here too: the NumPy twin rounds every operation

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                                   # the metric multiply must never fuse into a sum
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-Wno-unknown-warning-option",
    "-Wno-inline-asm",                                     # M0 on a clobber list is reserved: that is the point of listing it
]

# the host pass does not know the device-only target feature and says so once per kernel: not an error
_NOISE = "'-packed-fp32-ops' is not a recognized feature for this target"


def _run(cmd):
    proc = subprocess.run(cmd, cwd=CSRC, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if _NOISE not in l and "warning generated" not in l)
    return proc.returncode, out


def build(verbose: bool = True, jobs: int = 8) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    base = [hipcc] + HIPCC_FLAGS + os.environ.get("MP_EXTRA_FLAGS", "").split() + ["-I", INCLUDE, "-I", CSRC]
    sources = SOURCES + SYNTH_SOURCES
    objs = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in sources]
    cmds = [base + ["-x", "hip", "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(sources, objs)]
    if verbose:
        print(" ".join(cmds[0][:-6]) + " -x hip -c <each of " + " ".join(sources) + ">", flush=True)
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(cmds)))) as pool:
        results = list(pool.map(_run, cmds))
    failed = False
    for s, (rc, out) in zip(sources, results):
        if out.strip() and (verbose or rc):
            print(f"--- {s}\n{out}", flush=True)
        failed = failed or rc != 0
    if failed:
        raise RuntimeError("hipcc failed")
    for lib, part in ((LIB_PATH, objs[:len(SOURCES)]), (SYNTH_LIB_PATH, objs[len(SOURCES):])):
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + part + ["-o", lib]
        if verbose:
            print(" ".join(link), flush=True)
        rc, out = _run(link)
        if out.strip() and (verbose or rc):
            print(out, flush=True)
        if rc:
            raise RuntimeError(f"link failed with exit code {rc}")
    return LIB_PATH


if __name__ == "__main__":
    build()
    sys.exit(0)
