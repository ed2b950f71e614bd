"""Builds libgsd.so (the gfx950 HIP library behind include/gsd.h) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libgsd.so")
BENCH_LIB_PATH = os.path.join(PKG_DIR, "libgsd_bench.so")     # measurement aid of bench.py only

SOURCES = ["gsd_api.hip", "mask_build.hip", "accept_path.hip", "node_argmax.hip", "dag_attention_f32.hip",
           "dag_attention_bf16.hip", "unmerge_tree.hip", "commit_kv.hip", "accept_stochastic.hip", "build_graph.hip"]

# -no-hip-rt: the library carries no dependency on a particular libamdhip64; the process that loads it (the
# Python binding: the runtime torch already runs on) supplies the HIP runtime.  Two HIP runtimes in one process
# do not share devices, streams or pointers.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-no-hip-rt",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
               "-Wno-unused-command-line-argument"]


def build_library(verbose: bool = False, extra_flags: list[str] | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *(extra_flags or []), "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    cmd = [hipcc, *HIPCC_FLAGS, *(extra_flags or []), os.path.join(CSRC, "bench_mfma_loop.hip"), "-o", BENCH_LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
