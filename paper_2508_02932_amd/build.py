"""Builds libplora.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libplora.so")
BENCH_LIB = os.path.join(HERE, "libplora_bench.so")      # ceiling microkernels for bench.py, not the product
SOURCES = ["plora_api.hip", "small_kernels.hip", "f32_kernels.hip", "skinny_bf16.hip",
           "gemm_bf16.hip", "tokcontract_bf16.hip", "adamw.hip", "expand_bf16.hip", "nf4.hip",
           "planner.cpp"]                                     # host only: the packing planner
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src: str, obj_dir: str = OBJ, extra=()) -> str:
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and "argument unused during compilation" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES + ["bench_ceilings.hip"]))
    for lib, parts in ((LIB, objs[:-1]), (BENCH_LIB, objs[-1:])):
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *parts]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stderr)
        if verbose:
            print("built", lib)
    return LIB


def build_variant(lib_path: str, extra_flags, sources=("gemm_bf16.hip",)) -> str:
    """A copy of libplora.so at lib_path in which `sources` are compiled with extra flags (tuning runs; the other
    objects are taken from the last regular build)."""
    obj_dir = lib_path + ".obj"
    os.makedirs(obj_dir, exist_ok=True)
    objs = []
    for src in SOURCES:
        if src in sources:
            objs.append(_compile(src, obj_dir, tuple(extra_flags)))
        else:
            objs.append(os.path.join(OBJ, os.path.splitext(src)[0] + ".o"))
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path, *objs], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    return lib_path


if __name__ == "__main__":
    build(verbose=True)
