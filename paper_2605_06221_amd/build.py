"""Build libuniprefill.so (gfx950) in-tree with hipcc.  No JIT cache: the built
library sits next to this file so that it travels with the source tree."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libuniprefill.so")
PIPES_BENCH_PATH = os.path.join(HERE, "up_pipes_bench.exe")
SOURCES = ["up_api.hip", "up_copy.hip", "up_select.hip", "up_sweep.hip", "up_topp.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed-FP32 instructions are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # device code never sees NaN by contract (finite inputs); without this every fmaxf drags a
    # canonicalising v_max along.  Infinities are still honoured (masks use -inf).
    "-Xarch_device", "-fno-honor-nans",
    "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: cannot build libuniprefill.so")
    return exe


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles."""
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out, flush=True)
    cmd = [hipcc_path(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB_PATH, *objs]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}")
    build_pipes_bench(verbose)
    return LIB_PATH


def build_pipes_bench(verbose: bool = False) -> str:
    """The stand-alone measurement program of the matrix / vector pipes (not part of the library)."""
    flags = [f for f in HIPCC_FLAGS if f != "-fPIC"]
    cmd = [hipcc_path(), *flags, os.path.join(CSRC, "up_pipes_bench.hip"), "-o", PIPES_BENCH_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on up_pipes_bench.hip:\n{res.stdout}")
    return PIPES_BENCH_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
