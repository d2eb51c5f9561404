"""Build liblasad.so (hand-written HIP, gfx950 only) in-tree with hipcc.

Usage: ``python -m paper_2507_01652_amd.build``.  The library lands next to this
file so that it travels with the source tree; nothing is JIT-compiled at import.
"""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "liblasad.so")

SOURCES = [
    "lasad_api.hip",
    "lasad_decay.hip",
    "lasad_forward_generic.hip",
    "lasad_forward_scan.hip",
    "lasad_forward_mfma.hip",
    "lasad_forward_mfma_ws.hip",
    "lasad_forward_mfma_ws12.hip",
    "lasad_forward_gated_mfma.hip",
    "lasad_forward_gated_ws.hip",
    "lasad_decode.hip",
    "lasad_decode_cached.hip",
    "lasad_backward.hip",
    "lasad_backward_gated.hip",
    "lasad_backward_gated_mfma.hip",
    "lasad_backward_layer.hip",
]

# Packed-fp32 instruction selection is switched off for every HIP translation unit.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, extra_flags=(), jobs: int | None = None) -> str:
    """Compile every source to an object (several at a time) in a temporary folder, then link the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or max(1, min(8, os.cpu_count() or 1))
    with tempfile.TemporaryDirectory(prefix="lasad_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, src + ".o")
            cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
    print("built", LIB)
