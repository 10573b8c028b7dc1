"""Builds libmoehot.so (hand-written HIP for gfx950) in-tree with hipcc.

`python -m paper_2411_10003_amd.build` compiles every translation unit of csrc/ and links the
shared library next to this file.  hipcc cross-compiles, so no GPU is needed to build.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoehot.so")
UNITS = ["api", "gate", "gate_grad", "route", "rows", "plan", "ffn_f32", "ffn_bf16", "noalloc", "calib"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    # packed fp32 math is kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # "#pragma unroll" on loops that a compile-time variant of a kernel removes altogether
    "-Wno-pass-failed",
]


def _compile(unit: str) -> str:
    src = os.path.join(CSRC, unit + ".hip")
    obj = os.path.join(OBJ, unit + ".o")
    cmd = [HIPCC, *FLAGS, *os.environ.get("MOE_EXTRA_FLAGS", "").split(), "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {unit}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, UNITS))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
