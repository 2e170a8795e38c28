"""Build libq8.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libq8.so")
SOURCES = ["q8_api.hip", "q8_elementwise.hip", "q8_gemm.hip", "q8_embedding.hip",
           "q8_gemm_tile_256x256_w4.hip", "q8_gemm_tile_256x256_w8.hip", "q8_gemm_tile_128x128_w4.hip",
           "q8_gemm_tile_192x256_w4.hip", "q8_gemm_tile_192x256_w8.hip", "q8_gemm_tile_192x128_w4.hip", "q8_layernorm.hip", "q8_attention.hip", "q8_ceiling.hip", "q8_fc_small.hip"]
OBJ_DIR = os.path.join(HERE, "_build")

# -ffp-contract=off: the product x*S of Eq. 1 must be rounded on its own before the
# rounding step.  Packed fp32 instructions are switched off for the whole library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         "-I", INCLUDE, "-I", CSRC]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def build(verbose: bool = False) -> str:
    """Compile every translation unit (in parallel) and link libq8.so.  Always recompiles."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OBJ_DIR, exist_ok=True)
    cc = hipcc()
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [[cc, *FLAGS, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
