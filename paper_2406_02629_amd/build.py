"""Compile the HIP library for gfx950: paper_2406_02629_amd/libssnet.so over
p = 2^61 - 1 and, from the same sources with -DSS_FIELD_P45, libssnet_p45.so
over p = 2^45 - 55.

hipcc cross-compiles without a GPU.  Each .hip file is compiled to an object
and the objects are linked into one shared library per field that exports the
C ABI of include/ssnet.h.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libssnet.so")
LIB_P45 = os.path.join(HERE, "libssnet_p45.so")
VARIANTS = {"p61": (LIB, []), "p45": (LIB_P45, ["-DSS_FIELD_P45"])}
SOURCES = ["stream_kernels.hip", "gemm_kernels.hip", "ssnet_api.hip", "probes.hip"]
HEADERS = ["field.hpp", "kernels.hpp", "eval.hpp", "digits.hpp", os.path.join("..", "..", "include", "ssnet.h")]
# kernarg preload: the first kernel arguments arrive in scalar registers with the wave instead of by a load at its
# start, which is worth about half a microsecond on each of the short streaming launches of a batch-1 layer
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wall", "-Wno-unused-command-line-argument"]


def _newest_source() -> float:
    paths = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return max(os.path.getmtime(p) for p in paths)


def is_current() -> bool:
    newest = _newest_source()
    return all(os.path.exists(lib) and os.path.getmtime(lib) >= newest for lib, _ in VARIANTS.values())


def build(force: bool = True, verbose: bool = False) -> str:
    """Build both libraries; returns the path of the default one."""
    if not force and is_current():
        return LIB
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(job):
        tag, src = job
        obj = os.path.join(OBJ, src.replace(".hip", f".{tag}.o"))
        cmd = ["hipcc", *FLAGS, *VARIANTS[tag][1], "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src} ({tag}):\n{r.stdout}\n{r.stderr}")
        if verbose and r.stderr.strip():
            print(r.stderr, file=sys.stderr)
        return obj

    jobs = [(tag, src) for tag in VARIANTS for src in SOURCES]
    with ThreadPoolExecutor(max_workers=len(jobs)) as ex:
        objs = list(ex.map(compile_one, jobs))
    for v, tag in enumerate(VARIANTS):
        lib = VARIANTS[tag][0]
        # -Bsymbolic: references inside a library bind to that library, also when both are loaded globally
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-Bsymbolic", "-o", lib + ".tmp",
               *objs[v * len(SOURCES):(v + 1) * len(SOURCES)]]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed ({tag}):\n{r.stdout}\n{r.stderr}")
        os.replace(lib + ".tmp", lib)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
