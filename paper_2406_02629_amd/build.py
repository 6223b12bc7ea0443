"""Compile the HIP library for gfx950 into paper_2406_02629_amd/libssnet.so.

hipcc cross-compiles without a GPU.  Each .hip file is compiled to an object
and the objects are linked into one shared library that exports the C ABI of
include/ssnet.h.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libssnet.so")
SOURCES = ["stream_kernels.hip", "gemm_kernels.hip", "ssnet_api.hip"]
HEADERS = ["field.hpp", "kernels.hpp", "eval.hpp", "digits.hpp", os.path.join("..", "..", "include", "ssnet.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def _newest_source() -> float:
    paths = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return max(os.path.getmtime(p) for p in paths)


def is_current() -> bool:
    return os.path.exists(LIB) and os.path.getmtime(LIB) >= _newest_source()


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and is_current():
        return LIB
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        if verbose and r.stderr.strip():
            print(r.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp", *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
