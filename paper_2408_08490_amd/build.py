"""Builds libhgnn.so (host runtime + gfx950 kernels) in-tree with hipcc.

Every source is compiled to an object of its own (in parallel), then linked.  `build_library()` recompiles
everything; `build_library(incremental=True)` (or `python -m paper_2408_08490_amd.build -i`) skips objects that
are newer than their source and every header."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhgnn.so")
SOURCES = ["api.cpp", "host_build.cpp", "sampler.cpp", "noalloc.hip", "kernels_mem.hip", "kernels_spmm.hip", "kernels_gemm.hip", "kernels_gemm2.hip",
           "kernels_attn.hip", "kernels_optim.hip", "device_build.hip"]
FLAGS = ["-O3", "-std=c++20", "--offload-arch=gfx950", "-fPIC", "-Wno-inline-asm", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
NOISE = "packed-fp32-ops"


def hipcc_path():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def _headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(os.path.dirname(HERE), "include", "hgnn.h"))
    return hs


def _compile(src, obj, verbose):
    cmd = [hipcc_path()] + FLAGS + ["-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    return err


def build_library(verbose=True, incremental=False, jobs=8):
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in _headers())
    todo, objs = [], []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        objs.append(obj)
        fresh = incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header)
        if not fresh:
            todo.append((src, obj))
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(todo) or 1))) as ex:
        for err in ex.map(lambda a: _compile(a[0], a[1], verbose), todo):
            if verbose and err.strip():
                print(err)
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp"] + objs + ["-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    build_library(incremental="-i" in sys.argv[1:])
