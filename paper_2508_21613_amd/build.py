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
# CHM_SANITIZE=1: the HOST code of the library instrumented with AddressSanitizer and UndefinedBehaviorSanitizer
# (device code is compiled as always), as libchm_san.so; for the host-only tests, run with the sanitizer runtime
# loaded first:
#   CHM_SANITIZE=1 python -m paper_2508_21613_amd.build
#   CHM_SANITIZE=1 LD_PRELOAD=$(hipcc -print-file-name=libclang_rt.asan-x86_64.so) ASAN_OPTIONS=detect_leaks=0 \
#       python -m pytest tests/test_library_abi.py tests/test_guard_selection.py -q
# (the compiler's own runtime, which also carries the handlers of the undefined-behaviour checks)
SANITIZE = os.environ.get("CHM_SANITIZE", "") == "1"
OBJ = os.path.join(HERE, "_build_san" if SANITIZE else "_build")
LIB = os.path.join(HERE, "libchm_san.so" if SANITIZE else "libchm.so")
HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
                 "-Xarch_host", "-g"]
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
            todo.append(["hipcc"] + FLAGS + (HOST_SANITIZE if SANITIZE else []) + ["-x", "hip", "-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(todo)))) as pool:
        list(pool.map(run, todo))
    run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + (["-fsanitize=address,undefined", "-fno-gpu-sanitize", "-shared-libsan"] if SANITIZE else [])
        + objs + ["-o", LIB])
    return LIB


if __name__ == "__main__":
    build(changed_only="--changed" in sys.argv[1:])
    print("built", LIB)
