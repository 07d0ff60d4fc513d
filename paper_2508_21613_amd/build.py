"""Builds libchm.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2508_21613_amd.build            # compile every source, link
    python -m paper_2508_21613_amd.build --changed  # only the sources newer than their objects

Every source is compiled to an object of its own (in parallel), then linked.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libchm.so")
SOURCES = ["chm_host.cpp", "chm_pool.cpp", "chm_kernels.hip", "chm_fast.hip", "chm_replan.hip", "chm_probe.hip"]
# packed-FP32 instruction selection is switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]


def _headers_mtime():
    inc = os.path.join(os.path.dirname(HERE), "include")
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    files += [os.path.join(inc, f) for f in os.listdir(inc) if f.endswith(".h")]
    return max(os.path.getmtime(f) for f in files)


def build(verbose=True, changed_only=False):
    os.makedirs(OBJ, exist_ok=True)
    newest_header = _headers_mtime()
    todo, objs = [], []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        objs.append(obj)
        fresh = os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src), newest_header)
        if not (changed_only and fresh):
            todo.append(["hipcc"] + FLAGS + ["-x", "hip", "-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(todo)))) as pool:
        list(pool.map(run, todo))
    run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB])
    return LIB


if __name__ == "__main__":
    build(changed_only="--changed" in sys.argv[1:])
    print("built", LIB)
