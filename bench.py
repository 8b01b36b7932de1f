#!/usr/bin/env python3
"""Benchmark of the packed multi-LoRA linear layer (forward + backward) on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: plora_linear_fwd
followed by plora_linear_bwd on the Llama-3-8B-shaped q_proj configuration (d_in = d_out = 4096,
bf16, 4 adapters of rank 8/16/32/64 with 2048 tokens each), inputs resident in HBM.

Prints ONE JSON line: whole-step TFLOP/s (FLOPs = 4 T D K + 6 (D+K) sum(L r)), tokens/s, the
roofline of the dominant kernel (the forward base GEMM with the fused expand, timed with HIP events
on its own stream inside a second pass of the same steps), the other kernels' rates, and the fp64
CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E peak


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload configuration 1..5 (default: the headline one)")
    ap.add_argument("--linear", type=int, default=0, help="which linear of the configuration")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--sequential", action="store_true",
                    help="also time the same step issued one adapter per call (context figure; off by default so "
                         "that a profile of the default command only holds the packed kernels)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters when profiling this script)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2508_02932_amd import plora
    from paper_2508_02932_amd import workloads as wl
    import gpu_harness as gh

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    plora.lib()

    lin = wl.config(args.config)[args.linear]
    lay = lin.layout
    T, D, K = lay.T, lin.D, lin.K
    e = 2 if lin.dtype == "bf16" else 4
    t = lin.tensors()
    dp = gh.upload(lin, t)
    sum_Lr = lay.sum_Lr()
    R = int(sum(int(r) for r in lay.rank))
    flops = lin.flops_fwd_bwd()

    def step():
        plora.plora_linear_fwd(dp.desc, dp.x, dp.W, dp.A, dp.B, dp.y, dp.h, dp.ws)
        plora.plora_linear_bwd(dp.desc, dp.x, dp.W, dp.A, dp.B, dp.dy, dp.h, dp.dx, dp.dA, dp.dB, dp.ws)

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # spread of single steps (context; the metric above is the mean of the timed region): one event pair per step
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in evs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in evs)
    step_stats = {"median_ms": round(per_step[len(per_step) // 2], 4), "min_ms": round(per_step[0], 4),
                  "max_ms": round(per_step[-1], 4)}

    # second pass of the same steps with every kernel bracketed by HIP events on its stream
    plora.plora_set_kernel_timing(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    kern = {}
    for name in plora.KERNEL_CLASSES:
        ms, n = plora.plora_kernel_time(name)
        kern[name] = (ms / n) if n else None
    plora.plora_set_kernel_timing(False)

    # context leg (not the metric): the same work issued one adapter at a time, i.e. one forward and one
    # backward call per adapter on its own rows with a single-segment description - the launch pattern
    # that packing replaces (the paper's kernel tables compare against it)
    sequential = None
    if args.sequential and lay.n_adapters > 0 and all(int(a) >= 0 for a in lay.seg_adapter) \
            and len(set(int(a) for a in lay.seg_adapter)) == lay.n_seg:
        subs = []
        h_off = 0
        for sidx in range(lay.n_seg):
            k = int(lay.seg_adapter[sidx])
            lo, hi = int(lay.seg_off[sidx]), int(lay.seg_off[sidx + 1])
            L = hi - lo
            if L == 0:
                continue
            d = plora.Desc(L, D, K, np.array([0, L]), np.array([0]), np.array([lay.rank[k]]),
                           np.array([lay.scale[k]]), dp.desc.dtype)
            assert plora.plora_workspace_bytes(d) <= dp.ws.numel()
            n_h = L * int(lay.rank[k])
            subs.append((d, dp.x[lo:hi], dp.y[lo:hi], dp.dy[lo:hi], dp.dx[lo:hi], [dp.A[k]], [dp.B[k]],
                         [dp.dA[k]], [dp.dB[k]], dp.h[h_off:h_off + n_h]))
            h_off += n_h

        def seq_step():
            for d, x_, y_, dy_, dx_, A_, B_, dA_, dB_, h_ in subs:
                plora.plora_linear_fwd(d, x_, dp.W, A_, B_, y_, h_, dp.ws)
            for d, x_, y_, dy_, dx_, A_, B_, dA_, dB_, h_ in subs:
                plora.plora_linear_bwd(d, x_, dp.W, A_, B_, dy_, h_, dx_, dA_, dB_, dp.ws)

        n_seq = max(5, args.steps // 2)
        for _ in range(3):
            seq_step()
        torch.cuda.synchronize()
        t0s = time.perf_counter()
        for _ in range(n_seq):
            seq_step()
        torch.cuda.synchronize()
        seq_ms = (time.perf_counter() - t0s) * 1e3 / n_seq
        sequential = {"ms_per_step": round(seq_ms, 4), "steps": n_seq, "calls_per_step": 2 * len(subs),
                      "packed_speedup": round(seq_ms / ms_per_step, 3),
                      "note": "same library, one forward and one backward call per adapter on its own rows"}

    # algorithmic work per launch of each kernel (true ranks, nothing padded)
    alg = {
        "gemm_fwd": ("mfma", 2.0 * T * D * K + 2.0 * K * sum_Lr),
        "gemm_dx": ("mfma", 2.0 * T * D * K + 2.0 * D * sum_Lr),
        "shrink": ("hbm", T * D * e + D * R * e + sum_Lr * 4.0),
        "dh": ("hbm", T * K * e + R * K * e + sum_Lr * 4.0),
        "db": ("hbm", T * K * e + sum_Lr * 4.0 + R * K * 4.0),
        "da": ("hbm", T * D * e + sum_Lr * 4.0 + D * R * 4.0),
    }
    kernels = {}
    for name, (bound, work) in alg.items():
        ms = kern.get(name)
        if not ms:
            continue
        if bound == "mfma":
            a = work / (ms * 1e-3) / 1e12
            kernels[name] = {"ms": round(ms, 4), "bound": bound, "achieved": round(a, 1), "unit": "TFLOP/s",
                             "frac": round(a / PEAK_BF16_MFMA_TFLOPS, 4)}
        else:
            a = work / (ms * 1e-3) / 1e9
            kernels[name] = {"ms": round(ms, 4), "bound": bound, "achieved": round(a, 1), "unit": "GB/s",
                             "frac": round(a / PEAK_HBM_GBS, 4)}
    if kern.get("pack"):
        kernels["pack"] = {"ms": round(kern["pack"], 4)}
    # when the saved activation is handed to backward, class "shrink" of the last call is the
    # conversion kernel; the forward shrink is what the roofline entry should describe
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_config{args.config}_linear{args.linear}.txt")
    if os.path.exists(tpath):
        # committed summary of two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this script, already
        # scaled by the copy-kernel calibration; line format: "gemm_fwd <bytes per launch>"
        for line in open(tpath):
            parts = line.split()
            if len(parts) >= 2 and parts[0] == "gemm_fwd":
                traffic = float(parts[1])
    dom = kernels.get("gemm_fwd", {})
    roofline = {"kernel": "k_gemm<forward> (x W with fused scale*h*B_k)", "bound": "mfma",
                "achieved": dom.get("achieved"), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": dom.get("frac"), "traffic": traffic,
                "avg_launch_ms": dom.get("ms")}

    cpu = None
    if not args.no_cpu:
        import oracle
        from util import make_problem
        p = make_problem(oracle, lin, t)
        rng = np.random.default_rng(0)
        cores = oracle.loops.threads()

        def rows_time(n):
            rows = np.sort(rng.choice(T, size=min(n, T), replace=False))
            a = time.perf_counter()
            oracle.loops.fwd_rows(p, rows)
            oracle.loops.bwd_rows(p, t.dy, rows)
            return time.perf_counter() - a, len(rows)

        probe_s, probe_n = rows_time(2 * cores)
        n_rows = int(max(2 * cores, min(T, 12.0 / max(probe_s / probe_n, 1e-6))))
        rows_s, n_rows = rows_time(n_rows)
        # weight gradients: every adapter when that stays within a few seconds, else the largest-rank one
        k_big = int(np.argmax(lay.rank))
        Lr = [sum(int(lay.seg_off[s + 1] - lay.seg_off[s]) * int(lay.rank[k])
                  for s in range(lay.n_seg) if lay.seg_adapter[s] == k) for k in range(lay.n_adapters)]
        a = time.perf_counter()
        oracle.loops.grad_adapter(p, t.dy, k_big)
        one_s = time.perf_counter() - a
        done = [k_big]
        if one_s * (sum_Lr / max(Lr[k_big], 1)) < 15.0:
            for k in range(lay.n_adapters):
                if k != k_big and Lr[k] > 0:
                    oracle.loops.grad_adapter(p, t.dy, k)
                    done.append(k)
        grad_s = time.perf_counter() - a
        Lr_done = sum(Lr[k] for k in done)
        # whole-step estimate: row part scaled to T rows; weight-gradient part scaled by sum(L r)
        est_step_s = rows_s * (T / n_rows) + grad_s * (sum_Lr / max(Lr_done, 1))
        whole = n_rows == T and Lr_done == sum_Lr
        cpu = {"value": round(flops / est_step_s / 1e12, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
               "tokens_per_s": round(T / est_step_s, 2),
               "sample": f"fp64 scalar-loop oracle: y and dx of {n_rows} random rows of {T} ({rows_s:.1f} s) plus "
                         f"dA, dB of {len(done)} of {lay.n_adapters} adapters ({grad_s:.1f} s); "
                         + ("the whole step, nothing extrapolated" if whole else "whole step extrapolated")}

    out = {
        "metric": "packed multi-LoRA layer fwd+bwd TFLOP/s",
        "value": round(flops / (ms_per_step * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s",
        "tokens_per_s": round(T / (ms_per_step * 1e-3), 1),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "step_ms": step_stats,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if lin.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"config {args.config} / {lin.name}: d_in={D} d_out={K} T={T} "
                               f"adapters={lay.n_adapters} ranks={sorted(set(int(r) for r in lay.rank))}",
                   "tokens": T, "d_in": D, "d_out": K, "n_adapters": lay.n_adapters,
                   "flops_per_step": flops},
        "frac_of_bf16_mfma_peak": round(flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4),
        "roofline": roofline,
        "kernels": kernels,
        "sequential_adapters": sequential,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
