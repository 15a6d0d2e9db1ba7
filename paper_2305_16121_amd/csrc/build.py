"""Compile the sources of this directory (HIP kernels for gfx950, host C++) into liboases.so (in-tree, next to the package)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
PKG = os.path.dirname(HERE)
LIB = os.path.join(PKG, "liboases.so")
# (source, object stem, extra flags); gemm.hip is compiled once per contraction form so that its kernel instantiations build
# in parallel; planner.cc is host code only
SOURCES = (("gemm.hip", "gemm_nn", ["-DOASES_GEMM_PART=0"]), ("gemm.hip", "gemm_nt", ["-DOASES_GEMM_PART=1"]),
           ("gemm.hip", "gemm_tn", ["-DOASES_GEMM_PART=2"]), ("api.hip", "api", []), ("attention.hip", "attention", []),
           ("elementwise.hip", "elementwise", []), ("noalloc.hip", "noalloc", []), ("probe.hip", "probe", []), ("planner.cc", "planner", []))
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-fno-gpu-rdc"]


def _hipcc() -> str:
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.exists(c) or c == "hipcc":
            return c
    return "hipcc"


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def one(item):
        src, stem, flags = item
        obj = os.path.join(objdir, stem + ".o")
        cmd = [hipcc, *FLAGS, *flags, *(extra or []), "-c", os.path.join(HERE, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=9) as ex:
        objs = list(ex.map(one, SOURCES))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
