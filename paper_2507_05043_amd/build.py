"""Compile the HIP sources into libmolink_stage.so (in-tree, gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libmolink_stage.so")            # 16-bit element type bfloat16
LIB_PATH_F16 = os.path.join(HERE, "libmolink_stage_f16.so")    # the same sources with IEEE half elements
SOURCES = ("gemm.hip", "w4.hip", "elementwise.hip", "attention.hip", "stage.hip", "handoff.hip", "controller.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed fp32 instructions are switched off for every kernel of the library
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# The attention kernels rescale their MFMA accumulators with vector arithmetic at every step, so the
# accumulators must live in ordinary vector registers: in accumulation registers every rescaling costs a
# copy out and a copy back per register.
EXTRA_FLAGS = {"attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _compile(job: tuple) -> str:
    src, f16 = job
    obj = os.path.join(CSRC, src.replace(".hip", ".f16.o" if f16 else ".o"))
    cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), *(["-DMOLINK_F16"] if f16 else []), "-c",
           os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{res.stderr}")
    return obj


def _link(objs: list, path: str) -> None:
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", path]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")


def build(verbose: bool = False) -> str:
    """Compile every source for both element types and link the two shared libraries; returns the
    bfloat16 library's path."""
    jobs = [(src, f16) for f16 in (False, True) for src in SOURCES]
    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(_compile, jobs))
    _link(objs[:len(SOURCES)], LIB_PATH)
    _link(objs[len(SOURCES):], LIB_PATH_F16)
    if verbose:
        print("built", LIB_PATH, "and", LIB_PATH_F16, file=sys.stderr)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
