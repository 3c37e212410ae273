"""Builds libpipefill.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpipefill.so")
SOURCES = ["planner.cpp", "scheduler.cpp", "gemm_inst_a.hip", "gemm_inst_b.hip", "gemm_inst_c.hip", "gemm_inst_d.hip", "gemm.hip", "gemm_tn.hip", "elementwise.hip", "attention.hip", "attention_bwd.hip", "train_kernels.hip", "runtime.hip", "runtime_train.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = True, jobs: int = 8) -> str:
    """Compile every source and link the shared library; returns its path."""
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src + ".o")
        objs.append(obj)
        cmd = ["hipcc", *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _wait(procs, verbose)
    _wait(procs, verbose)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if out.returncode != 0:
        raise RuntimeError("link failed:\n" + out.stdout)
    if verbose:
        print("built", LIB)
    return LIB


def _wait(procs, verbose):
    while procs:
        src, p = procs.pop(0)
        text = p.communicate()[0]
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"compiling {src} failed:\n{text}")
        if verbose and text.strip():
            print(f"[{src}]\n{text}")


if __name__ == "__main__":
    build()
    sys.exit(0)
