"""Builds libsparse_set.so (gfx950) from csrc/*.hip with hipcc, in-tree.

`python -m paper_2102_01732_amd.build --gather-ceiling` also builds the stand-alone random-row-gather
microbenchmark (csrc/gather_ceiling.hip -> paper_2102_01732_amd/gather_ceiling), which measures the rate the
sparse kernels are held against; the library does not use it and build() does not compile it."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsparse_set.so")
SOURCES = ["sl_api.hip", "sl_train.hip", "sl_topology.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wno-unused-result"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_gather_ceiling() -> str:
    out = os.path.join(HERE, "gather_ceiling")
    r = subprocess.run(["hipcc", *FLAGS, os.path.join(CSRC, "gather_ceiling.hip"), "-o", out], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for gather_ceiling.hip:\n" + r.stderr)
    return out


def build(verbose: bool = False) -> str:
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    if "--gather-ceiling" in sys.argv[1:]:
        print("built", build_gather_ceiling())
