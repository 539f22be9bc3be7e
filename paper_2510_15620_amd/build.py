"""Compile the HIP library for gfx950: python -m paper_2510_15620_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libprism.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

SOURCES = ["prism_api.hip", "elementwise.hip", "prune.hip", "gemm_fp32.hip", "gemm_16.hip", "attn_fp32.hip",
           "attn_16.hip", "quant.hip"]
# PRISM_EXTRA_FLAGS: extra hipcc flags for experiments (e.g. -D switches of timing builds); empty in normal use
COMMON = ["--offload-arch=gfx950", "-O3", *os.environ.get("PRISM_EXTRA_FLAGS", "").split(), "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          # hipcc -O3 may otherwise form packed-fp32 instructions from ordinary float code
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the pruning decisions must reproduce a fixed fp64 operation order: no fused multiply-add
EXTRA = {"prune.hip": ["-ffp-contract=off"]}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *COMMON, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
