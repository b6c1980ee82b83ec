"""Builds libgpga.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to build."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libgpga.so")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
SOURCES = ["gpga_api.hip", "gpga_step.hip", "gpga_mix.hip", "gpga_graph.hip", "gpga_grad.hip", "gpga_reduce.hip",
           "gpga_static.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-fno-gpu-rdc",
    # packed-FP32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; libgpga needs the ROCm toolchain to build")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 target feature and says so once per file: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if err.strip() and (verbose or res.returncode != 0):
        sys.stderr.write(err + "\n")
    if res.stdout and (verbose or res.returncode != 0):
        sys.stdout.write(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))


def build_library(verbose: bool = True) -> str:
    """Compile all HIP sources (one hipcc process per file, side by side) and link them into
    paper_2105_09080_amd/libgpga.so; returns its path.  Every call compiles everything."""
    extra = os.environ.get("GPGA_EXTRA_HIPCC_FLAGS", "").split()
    hipcc = hipcc_path()
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[hipcc, *HIPCC_FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
             os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-fno-gpu-rdc", "-shared", "-fPIC", *objs, "-o", LIB_PATH + ".tmp"], verbose)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


HOST_CHECK_PATH = os.path.join(OBJ_DIR, "gpga_host_check")


def build_host_check(verbose: bool = True) -> str:
    """The host-only check program (graph builders, validation of W, beta, schedule arithmetic) compiled from
    the library's own sources with AddressSanitizer and UndefinedBehaviorSanitizer on the host side.  Runs on
    the CPU; returns the path of the executable."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    cmd = [hipcc_path(), "-x", "hip", "--cuda-host-only", "-std=c++17", "-O1", "-g",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "gpga_graph.hip"), os.path.join(CSRC, "gpga_host_check.cpp"), "-o", HOST_CHECK_PATH]
    _run(cmd, verbose)
    return HOST_CHECK_PATH


if __name__ == "__main__":
    print(build_library())
