"""Builds libgemm_lineage.so (HIP, gfx950 only) next to this file.

Each .hip translation unit is compiled to an object in ``_build/`` and linked with
``hipcc -shared``.  Objects are rebuilt when their source or a header is newer, unless
``force`` is set.  hipcc cross-compiles without a GPU present.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgemm_lineage.so")
SOURCES = ["gemm_api.hip", "conv_api.hip", "topk.hip", "k0_naive.hip", "k123_valu_tiled.hip", "k4_mfma.hip", "probes.hip"]
HEADERS = [os.path.join(CSRC, "common.hpp"), os.path.join(CSRC, "k4_kernels.hpp"),
           os.path.join(os.path.dirname(HERE), "include", "gemm_lineage.h"),
           os.path.join(os.path.dirname(HERE), "include", "conv_lineage.h"),
           os.path.join(os.path.dirname(HERE), "include", "topk_lineage.h")]
# packed fp32 VALU forms (v_pk_*_f32) are switched off: the compiler must not form them for this target
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(p) for p in [path] + HEADERS)
    if force or not os.path.exists(obj) or os.path.getmtime(obj) < newest:
        r = subprocess.run(["hipcc", *FLAGS, "-c", path, "-o", obj], capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip():
            sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
