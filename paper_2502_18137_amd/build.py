"""Builds libsparge.so (gfx950) in-tree with hipcc.  `python -m paper_2502_18137_amd.build`."""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsparge.so")
OBJ_DIR = os.path.join(PKG, "_build")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"),
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-fhip-fp32-correctly-rounded-divide-sqrt", "-Wall", "-Wno-unused-function"]
# file -> extra flags.  The quantizer's fp32 operation sequence is part of the numerical contract:
# no fused multiply-add may be formed there.
SOURCES = {
    "stats_quant.hip": ["-ffp-contract=off"],
    "predict.hip": ["-ffp-contract=off"],
    "attn.hip": [],
    "v_fp8.hip": ["-ffp-contract=off"],
    "metrics.hip": ["-ffp-contract=off"],
    "permute.hip": [],
    "api.hip": [],
}


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = True) -> str:
    hipcc = _hipcc()
    os.makedirs(OBJ_DIR, exist_ok=True)
    # the attention loop's assembly is generated: rewrite it so that it cannot lag behind its generator
    r = subprocess.run([sys.executable, os.path.join(CSRC, "gen_attn_loop.py")], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gen_attn_loop.py failed:\n{r.stdout}\n{r.stderr}")

    def compile_one(item):
        src, extra = item
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
        return obj, warn

    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(compile_one, SOURCES.items()))
    for obj, warn in results:
        if verbose and warn:
            print(warn, file=sys.stderr)
    objs = [o for o, _ in results]
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build_library()
