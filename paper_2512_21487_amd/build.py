"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libmoe_ep.so")
OBJDIR = os.path.join(HERE, "_build")

SOURCES = ["router.hip", "dispatch.hip", "combine.hip", "transfer.hip", "grouped_gemm.hip", "schedule.hip", "dep_schedule.hip", "moe_ep.hip"]
# the benchmark's measurement aid: a library of its own, not linked into the layer's
PROBE_SOURCE = "probe.hip"
PROBE_LIB = os.path.join(HERE, "libmoe_ep_probe.so")
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 code generation is switched off on purpose (silent wrong results were seen
    # with some of its forms on this hardware generation)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the GEMM's K step is one fully unrolled sequence of up to 128 matrix instructions with their loads and
    # fragment reads; past the default threshold the compiler keeps a loop and the accumulators go to scratch memory
    "-mllvm", "-pragma-unroll-threshold=200000",
    "-I", INCLUDE, "-I", CSRC,
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJDIR, src.replace(".hip", ".o"))
    cmd = ["hipcc", *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    noise = "is not a recognized feature for this target"
    for line in (res.stdout + res.stderr).splitlines():
        if noise not in line and line.strip():
            sys.stderr.write(line + "\n")
    return obj


def build(verbose: bool = False) -> str:
    """Compile every source and link libmoe_ep.so next to this file. Always recompiles."""
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        objs = list(ex.map(_compile, SOURCES + [PROBE_SOURCE]))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs[:-1]])
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB, objs[-1]])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
