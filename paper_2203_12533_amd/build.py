"""Builds libpw.so (the HIP kernels + C boundary) in-tree with hipcc for gfx950.

Usage: python -m paper_2203_12533_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpw.so")
SOURCES = ["model_common.hip", "elementwise.hip", "norm.hip", "embed_xent.hip", "attention.hip", "attention_mfma.hip", "attention_dma.hip", "gemm.hip", "gemm_ring.hip",
           "lm.hip", "encdec.hip", "runtime.hip", "runtime_sched.hip", "runtime_models.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-result", "-Wno-inline-asm"]


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    srcp = os.path.join(CSRC, src)
    deps = [srcp] + [os.path.join(CSRC, h) for h in os.listdir(CSRC) if h.endswith(".hpp")] + \
           [os.path.join(HERE, "..", "include", "pw.h")]
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) > os.path.getmtime(d) for d in deps):
        return obj
    r = subprocess.run(["hipcc"] + FLAGS + ["-c", srcp, "-o", obj], capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


DISPATCH_BENCH = os.path.join(HERE, "tools", "dispatch_bench")


def build_tools() -> str:
    """The pure-C++ dispatch benchmark: host code only, talks to libpw.so through include/pw.h."""
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-I", os.path.join(HERE, "..", "include"),
                           os.path.join(HERE, "tools", "dispatch_bench.cpp"), "-L", HERE, "-lpw",
                           "-Wl,-rpath,$ORIGIN/..", "-Wl,-rpath,/opt/rocm/lib", "-o", DISPATCH_BENCH])
    return DISPATCH_BENCH


def build(force: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    build_tools()
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
