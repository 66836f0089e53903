"""Builds libtaskkv.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libtaskkv.so")
SOURCES = ["api.hip", "score_mfma64.hip", "score_screen.hip", "score_i8.hip", "score_i8_own.hip", "select.hip", "select_multi.hip", "cache.hip", "decode.hip", "decode_stream.hip"]
# packed-fp32 instructions are switched off on purpose (device pass only; the
# host pass prints a harmless "not a recognized feature" note)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature",
         "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _compile(src: str, obj: str) -> None:
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")


def build_library(verbose: bool = True) -> str:
    """Compile every HIP source and link libtaskkv.so next to this file."""
    bdir = os.path.join(PKG, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]
    with cf.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        list(ex.map(_compile, SOURCES, objs))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}", file=sys.stderr)
    return LIB


def build_c_caller(verbose: bool = True) -> str:
    """Compile tests/c_caller/taskkv_c_caller.c with gcc, as C, against the
    header and the library: the test program that calls the C ABI with no
    Python or C++ in between."""
    src = os.path.join(ROOT, "tests", "c_caller", "taskkv_c_caller.c")
    exe = os.path.join(ROOT, "tests", "c_caller", "taskkv_c_caller")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-O1", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"), src,
           "-L", PKG, "-ltaskkv", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2501_15113_amd", f"-Wl,-rpath,{os.path.join(rocm, 'lib')}", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gcc failed on the C caller:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {exe}", file=sys.stderr)
    return exe


if __name__ == "__main__":
    build_library()
    build_c_caller()
