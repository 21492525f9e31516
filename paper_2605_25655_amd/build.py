"""Build libthi.so and the benchmark's libthi_probe.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2605_25655_amd.build

hipcc cross-compiles without a GPU, so this also works on a CPU-only host.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libthi.so")
PROBE_LIB = os.path.join(PKG, "libthi_probe.so")      # measurement probes: not part of the product library
SOURCES = ["api.hip", "plan.hip", "skinny.hip", "rowslab.hip", "rowblock.hip", "attention.hip", "gemm.hip"]
PROBE_SOURCES = ["probes.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # leading scalar kernel arguments arrive preloaded in registers (the decode kernels pass the operands
    # of their first loads that way)
    "-mllvm", "-amdgpu-kernarg-preload-count=12",
]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    every = SOURCES + PROBE_SOURCES
    with ThreadPoolExecutor(max_workers=len(every)) as pool:
        objs = dict(zip(every, pool.map(_compile, every)))
    for lib, sources in ((LIB, SOURCES), (PROBE_LIB, PROBE_SOURCES)):
        cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib] + [objs[s] for s in sources]
        subprocess.check_call(cmd)
        if verbose:
            print(f"built {lib}")
    return LIB


if __name__ == "__main__":
    build()
