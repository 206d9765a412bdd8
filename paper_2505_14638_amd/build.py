"""Builds the C-ABI library libw4a8.so for gfx950 with hipcc, in-tree (next to this file)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libw4a8.so")
SOURCES = ["api.hip", "quantize_act.hip", "pack_weights.hip", "linear_canonical.hip", "linear_skinny.hip",
           "linear_mfma.hip", "linear_mfma2d.hip", "silu_mul.hip", "probe.hip", "dpq.hip", "hessian_factor.hip"]
# packed fp32 instructions are switched off for all device code (scalar fp32 only)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# linear_mfma.hip orders MFMAs, LDS reads and ALU work step by step; the backend's sinking pass otherwise moves the MFMAs
# of the modes that accumulate inside the matrix unit past the branches of a pass to its end, where all of the pass's
# activation operands are live at once and spill
# dpq.hip: Alg. 1 is specified as a sequence of single float32 operations (its integer decisions must be reproducible
# bit for bit), so a product must never be contracted with the sum or difference that consumes it
EXTRA_FLAGS = {"linear_mfma.hip": ["-mllvm", "-disable-machine-sink"],
               "linear_mfma2d.hip": ["-mllvm", "-disable-machine-sink"], "dpq.hip": ["-ffp-contract=off"]}


def build(verbose: bool = False) -> str:
    """Compile every HIP source and link libw4a8.so; always recompiles. Returns the library path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "is not a recognized feature" not in l)
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
