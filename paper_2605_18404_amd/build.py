"""Builds libmlip.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libmlip.so")
# (source, object name, extra flags); the equivariant model is compiled once per (l_max, phase) plus once for its interface
# functions: nine objects, side by side (the heaviest first)
SOURCES = [("equivariant.hip", f"equivariant_l{l}_p{ph}", [f"-DMLIP_EQV_LMAX={l}", f"-DMLIP_EQV_PHASE={ph}"])
           for l in (3, 2) for ph in (3, 2, 1, 0)] + \
          [("equivariant.hip", "equivariant_api", ["-DMLIP_EQV_PHASE=-1"]),
           ("model.hip", "model", []), ("api.hip", "api", []), ("graph.hip", "graph", []), ("graph_static.hip", "graph_static", []),
           ("optimizer.hip", "optimizer", []), ("gars.cpp", "gars", [])]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# The neighbour search decides r < r_c in fp32 and must take the same decision as a plain
# multiply-then-add evaluation: no fused multiply-add there.  The model kernels may fuse.
NO_FMA = {"graph.hip"}


def _compile(item) -> str:
    src, name, extra = item
    obj = os.path.join(HERE, "_build", name + ".o")
    os.makedirs(os.path.dirname(obj), exist_ok=True)
    contract = "-ffp-contract=off" if src in NO_FMA else "-ffp-contract=fast"
    cmd = ["hipcc", *FLAGS, *extra, contract, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build(verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=max(1, min(8, os.cpu_count() or 1))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {OUT}")
    return OUT


if __name__ == "__main__":
    build()
    sys.exit(0)
