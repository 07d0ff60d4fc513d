"""Builds libchm.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2508_21613_amd.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libchm.so")
SOURCES = ["chm_host.cpp", "chm_pool.cpp", "chm_kernels.hip", "chm_fast.hip", "chm_replan.hip", "chm_probe.hip"]
# packed-FP32 instruction selection is switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]


def build(verbose=True):
    flags = list(FLAGS)
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = ["hipcc"] + flags + ["-x", "hip"] + srcs + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
