"""Build libfedhybrid.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc.

Cross-compiles without a GPU.  Run as `python -m paper_2510_11400_amd.build`.
Every call compiles every source (one hipcc process per file, side by side) and links.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfedhybrid.so")
SOURCES = ("fh_abi.hip", "fh_compress.hip", "fh_decompress.hip", "fh_classify.hip", "fh_mixed.hip", "fh_sparse.hip",
           "fh_huffman.hip", "fh_chain.hip")

# Strict binary32 semantics on the device: no contraction (the one fused multiply-add
# of the method is written explicitly), IEEE division, denormals kept.  Packed-fp32
# instruction selection is disabled.
FLAGS = [
    "-std=c++17", "-O3", "--offload-arch=gfx950", "-fPIC",
    "-ffp-contract=off", "-fno-fast-math",
    "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]
_NOISE = "is not a recognized feature for this target"


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; ROCm is required to build libfedhybrid.so")
    return exe


def _run(cmd, verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, cwd=CSRC, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if _NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}): {' '.join(cmd)}\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose: bool = False, extra_flags=(), out: str = LIB, only=None) -> str:
    """Compile the sources (all of them, or those named in `only`, reusing the other objects)
    and link `out`."""
    os.makedirs(OBJ, exist_ok=True)
    exe = hipcc()
    objs = {s: os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES}
    todo = [s for s in SOURCES if only is None or s in only or not os.path.exists(objs[s])]
    jobs = min(len(todo), max(1, min(16, os.cpu_count() or 1)))
    if todo:
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda s: _run([exe, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, s), "-o", objs[s]],
                                         verbose), todo))
    _run([exe, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", out, *[objs[s] for s in SOURCES]], verbose)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True, only=sys.argv[1:] or None))
