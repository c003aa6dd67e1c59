"""Builds libcpoconv.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcpoconv.so")
SOURCES = ["capi.cpp", "encode.hip", "spmv_conv.hip", "spmv_conv_tile.hip", "spmv_conv_strip.hip", "spmv_conv_runs.hip", "im2col_gemm.hip"]

COMPILE_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept off (plain v_fma_f32 only)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Per-source flags.  The column-run kernel selects one of many code paths per NZE, each adding into
# its own accumulator registers; merging the common tails of those paths would turn the register
# numbers into run-time indices and move the accumulators to scratch memory.
EXTRA_FLAGS = {"spmv_conv_runs.hip": ["-mllvm", "-simplifycfg-sink-common=false"]}


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the packed-fp32 feature and says so: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(verbose: bool = False) -> str:
    """Compile every source to an object (in parallel) and link libcpoconv.so."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    jobs = []
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        jobs.append((obj, [hipcc] + COMPILE_FLAGS + EXTRA_FLAGS.get(src, []) +
                     ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]))
    if verbose:
        for _, cmd in jobs:
            print(" ".join(cmd), flush=True)
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        outs = list(pool.map(lambda j: _run(j[1]), jobs))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [o for o, _ in jobs] + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    outs.append(_run(link))
    if verbose:
        for o in outs:
            if o.strip():
                print(o)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
