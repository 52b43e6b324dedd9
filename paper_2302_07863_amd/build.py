"""Builds libbild.so (the HIP library behind include/bild.h) in-tree for gfx950.

Every translation unit is compiled to an object under `_build/` by its own hipcc
process (they run side by side), then the objects are linked into the library.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libbild.so")
# (source, object name, extra defines)
UNITS = [
    ("kernels.hip", "kernels.o", []),
    ("gemm_pre.hip", "gemm_pre.o", []),
    ("gemm_dense.hip", "gemm_dense.o", []),
    ("attention.hip", "attention.o", []),
    ("policy.hip", "policy.o", []),
    ("bild_api.hip", "bild_api.o", []),
    ("head_stats.hip", "head_stats.o", []),
    ("bench_api.hip", "bench_api.o", []),
    ("layout.cpp", "layout.o", []),
]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-pthread",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # leading scalar kernel parameters arrive in scalar registers at wave start (see BILD_GEMM_HOT_PARAMS)
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wno-unused-result", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _clean(text: str) -> str:
    return "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    procs = []
    extra = os.environ.get("BILD_EXTRA_DEFS", "").split()  # experiments: extra -D flags for every unit
    for src, obj, defs in UNITS:
        cmd = ["hipcc"] + FLAGS + defs + extra + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", os.path.join(OBJ, obj)]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = []
    for src, p in procs:
        out = _clean(p.communicate()[0])
        if p.returncode != 0:
            failed.append(f"{src}:\n{out}")
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed:\n" + "\n".join(failed))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread"] + \
          [os.path.join(OBJ, obj) for _, obj, _ in UNITS] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + _clean(r.stdout))
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
