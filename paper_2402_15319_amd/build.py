"""Builds libvq.so (HIP, gfx950 only) in-tree with hipcc.

Usage: python -m paper_2402_15319_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libvq.so")
OBJ_DIR = os.path.join(HERE, "_build")   # object files (kept out of the history)
BENCH_LIB_PATH = os.path.join(HERE, "libvq_bench.so")   # the benchmark's read probe, not part of the product
BENCH_SOURCES = ["vq_bench_probe.hip"]
SOURCES = ["vq_api.hip", "vq_pack.hip", "vq_decode.hip", "vq_gemv.hip", "vq_gemv_lora.hip", "vq_gemv_d4.hip", "vq_gemm.hip", "vq_em.hip"]
# packed-fp32 code generation is switched off on purpose for this machine pool
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def _link(sources, out, verbose):
    """Compiles every source to an object file (in parallel, one hipcc per file) and links them."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in sources]
    cmds = [[hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(sources, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs], verbose)


def build(verbose: bool = False) -> str:
    """Compiles libvq.so (the product) and libvq_bench.so (the benchmark's read probe)."""
    _link(SOURCES, LIB_PATH, verbose)
    _link(BENCH_SOURCES, BENCH_LIB_PATH, verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
