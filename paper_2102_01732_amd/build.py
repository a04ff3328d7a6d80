"""Builds libsparse_set.so (gfx950) from csrc/*.hip with hipcc, in-tree, and the stand-alone
gather-ceiling microbenchmark beside it."""
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
TOOL_SRC, TOOL = "gather_ceiling.hip", os.path.join(HERE, "gather_ceiling")
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


def _tool() -> None:
    cmd = ["hipcc", *FLAGS, os.path.join(CSRC, TOOL_SRC), "-o", TOOL]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {TOOL_SRC}:\n" + "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l))


def build(verbose: bool = False) -> str:
    with ThreadPoolExecutor(max_workers=len(SOURCES) + 1) as ex:
        tool = ex.submit(_tool)
        objs = list(ex.map(_compile, SOURCES))
        tool.result()
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
