"""Sweep of the placement of the base GEMM's loops inside the 32-byte instruction-fetch windows.

The GEMM kernel pads the instruction stream in front of its loops with PLORA_GEMM_PAD_FWD / PLORA_GEMM_PAD_DX
4-byte no-ops behind a 256-byte boundary (csrc/gemm_bf16.hip explains why that matters).  The best counts move
whenever the code behind the padding changes; this script builds the eight candidates and times both forms on a
workload, so that the defaults in the source can be set again.  Needs a GPU.

    python -m paper_2508_02932_amd.sweep_placement [--config 5 --linear 1 --steps 6]
    (--build-only / --time-only split the two halves, e.g. to compile on a machine without a GPU)
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys

from . import build as B


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--linear", type=int, default=1)
    ap.add_argument("--steps", type=int, default=6)
    ap.add_argument("--rounds", type=int, default=2, help="passes over the candidates (the chip warms up during a pass)")
    ap.add_argument("--build-only", action="store_true")
    ap.add_argument("--time-only", action="store_true")
    args = ap.parse_args()
    if not args.time_only:
        B.build()
    out_dir = os.path.join(B.OBJ, "placement")
    os.makedirs(out_dir, exist_ok=True)
    bench = os.path.join(B.ROOT, "bench.py")
    libs = []
    for n in range(8):
        lib = os.path.join(out_dir, f"libplora_pad{n}.so")
        if not args.time_only:
            B.build_variant(lib, [f"-DPLORA_GEMM_PAD_FWD={n}", f"-DPLORA_GEMM_PAD_DX={n}"])
        libs.append(lib)
    if args.build_only:
        return
    fwd = [[] for _ in libs]
    dx = [[] for _ in libs]
    for rnd in range(args.rounds):
        for n, lib in enumerate(libs):
            env = dict(os.environ, PLORA_LIBRARY=lib)
            res = subprocess.run([sys.executable, bench, "--no-cpu", "--no-per-config", "--no-context", "--config", str(args.config),
                                  "--linear", str(args.linear), "--steps", str(args.steps), "--warmup", "2"],
                                 env=env, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError(res.stderr[-2000:])
            k = json.loads(res.stdout.strip().splitlines()[-1])["kernels"]
            fwd[n].append(k["gemm_fwd"]["ms"])
            dx[n].append(k["gemm_dx"]["ms"])
            print(f"pass {rnd} pad {n}: forward GEMM {fwd[n][-1]:.4f} ms   dX GEMM {dx[n][-1]:.4f} ms", flush=True)
    mean = lambda v: sum(v) / len(v)
    print("means:", " ".join(f"{n}: {mean(fwd[n]):.3f}/{mean(dx[n]):.3f}" for n in range(8)))
    print("best: PLORA_GEMM_PAD_FWD =", min(range(8), key=lambda n: mean(fwd[n])), "  PLORA_GEMM_PAD_DX =",
          min(range(8), key=lambda n: mean(dx[n])))


if __name__ == "__main__":
    main()
