"""Builds paper_2605_10886_amd/libloka.so from csrc/*.hip with hipcc for gfx950.

    python -m paper_2605_10886_amd.build

Objects go to _build/ at the repository root (git-ignored); the shared library is
written next to this file so it travels with the tree.  hipcc cross-compiles, no
GPU is needed to build.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libloka.so")
SOURCES = ["api.hip", "quantize.hip", "gemm.hip", "gemm_panel32.hip", "gemm_wreg.hip", "gemm_strip.hip", "probe.hip", "dispatch.hip", "tracker.hip", "ceiling.hip"]

# -packed-fp32-ops off: packed fp32 VALU forms are kept out of the generated code.
# No fast-math: divisions and square roots stay correctly rounded, no FMA contraction
# across statements that the oracle treats as separate roundings.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


# Per-source additions.  gemm_panel32.hip: the main loop's instruction order is pinned with scheduling barriers,
# which bind the scheduler but not the machine-code sinking pass that runs before it; that pass moves the SCALED
# matrix instructions (which it takes for freely movable) out of their slots to the end of the loop body, behind
# every LDS read, and the accumulators spill.  The pass is switched off for that file (its other kernels come out
# the same, instruction for instruction, apart from a few address computations).
EXTRA_FLAGS = {"gemm_panel32.hip": ["-mllvm", "-disable-machine-sink"]}


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
