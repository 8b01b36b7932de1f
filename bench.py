#!/usr/bin/env python3
"""Benchmark of the packed multi-LoRA linear layer (forward + backward) on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: plora_linear_fwd
followed by plora_linear_bwd, inputs resident in HBM.  The headline workload is the largest
single-GPU configuration: the 70B-shaped MLP up projection (configuration 5, second linear:
d_in = 8192, d_out = 28672, 32768 tokens, 32 adapters of rank 8..128 in unequal segments).

Prints ONE JSON line:
  value / tokens_per_s  whole-step rate of the headline workload; FLOPs = 4 T D K + 6 (D+K) sum(L r)
  roofline              the dominant kernel (forward base GEMM with the fused expand): algorithmic FLOPs /
                        average launch duration, HIP events on the call's own stream (library timing hook)
  kernels               every kernel class the same way: GEMMs against the bf16 MFMA peak, the streaming
                        kernels (shrink, dH, dB, dA) as algorithmic bytes / time against the HBM peak; both
                        also as a fraction of the ceilings measured in this run (plain streaming read,
                        MFMA-only loop)
  per_config            the other configurations: 2, 3 (both linears), 4 (seven linears of a decoder layer,
                        forward in order then backward in reverse on one stream, with the total), 5 (attention),
                        each also replayed from a HIP graph; then the headline linear with W stored the other
                        way round and with W kept in both layouts
  lora_only             plora_lora_fwd / plora_lora_bwd on the headline workload (in-place update kernel)
  nf4_base              the headline step on a 4-bit NF4 base weight (expansion kernel, slowdown)
  cpu_baseline          the fp64 oracle on a bounded sample of the headline workload, on the host cores
Inputs of a step rotate over enough distinct sets of x / dy (more than 512 MB of them) that no kernel
finds its input in the 256 MB last-level cache from the step before.
"""
import argparse
import ctypes as C
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
ROTATE_BYTES = 600 << 20           # distinct input bytes a kernel sees before a buffer comes round again


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="workload configuration 1..5 (default: the headline one)")
    ap.add_argument("--linear", type=int, default=1,
                    help="which linear of the configuration; -1 with --config 4: the seven linears in sequence "
                         "(profiling runs; prints a short JSON line of its own)")
    ap.add_argument("--w-layout", choices=["in_out", "out_in", "both"], default="in_out",
                    help="storage of the frozen weight for the headline run: W[d_in][d_out] (default), W[d_out][d_in], or "
                         "both copies (forward reads [d_out][d_in], backward [d_in][d_out])")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--grouped", action="store_true",
                    help="with --config 4 --linear -1: q / k / v and gate / up as grouped calls (plora_group_fwd / _bwd)")
    ap.add_argument("--no-per-config", action="store_true", help="skip the per_config array (profiling runs)")
    ap.add_argument("--no-context", action="store_true", help="skip the ceilings and the vendor-GEMM context figures")
    ap.add_argument("--sequential", action="store_true",
                    help="also time the same step issued one adapter per call (context figure)")
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

    # ---- measured ceilings (bench-side library, not the product) -----------------------------------
    ceil = {"stream_read_gbs": None, "mfma_only_tflops": None, "mfma_only_constant_operands_tflops": None}
    if not args.no_context:
        blib_path = os.path.join(ROOT, "paper_2508_02932_amd", "libplora_bench.so")
        if os.path.exists(blib_path):
            bl = C.CDLL(blib_path)
            buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
            sink = torch.zeros(4, dtype=torch.float32, device="cuda")
            v = C.c_double(0)
            st = int(torch.cuda.current_stream().cuda_stream) or None
            if bl.plora_bench_stream_read(C.c_void_p(buf.data_ptr()), C.c_size_t(buf.numel()), 5,
                                          C.c_void_p(sink.data_ptr()), C.c_void_p(st), C.byref(v)) == 0:
                ceil["stream_read_gbs"] = round(v.value, 1)
            if bl.plora_bench_mfma_only(C.c_void_p(sink.data_ptr()), C.c_float(40.0), 1, C.c_void_p(st), C.byref(v)) == 0:
                ceil["mfma_only_tflops"] = round(v.value, 1)        # random operands: the ceiling for real data
            if bl.plora_bench_mfma_only(C.c_void_p(sink.data_ptr()), C.c_float(40.0), 0, C.c_void_p(st), C.byref(v)) == 0:
                ceil["mfma_only_constant_operands_tflops"] = round(v.value, 1)
            del buf, sink
            torch.cuda.empty_cache()

    def gpu_tensors(lin, seed):
        """Synthetic inputs of a linear drawn on the device (same distributions as workloads.py)."""
        lay = lin.layout
        g = torch.Generator(device="cuda").manual_seed(seed)
        dt = torch.bfloat16
        D, K, T = lin.D, lin.K, lay.T
        x = torch.randn(T, D, device="cuda", generator=g).to(dt)
        W = (torch.randn(D, K, device="cuda", generator=g) * (1.0 / D ** 0.5)).to(dt)
        dy = torch.randn(T, K, device="cuda", generator=g).to(dt)
        A = [((torch.rand(D, int(r), device="cuda", generator=g) * 2 - 1) * (1.0 / D ** 0.5)).to(dt) for r in lay.rank]
        B = [(torch.randn(int(r), K, device="cuda", generator=g) * (lin.var_B ** 0.5)).to(dt) for r in lay.rank]
        return x, W, dy, A, B

    class Runner:
        """One linear on the device with rotating input sets; step(i) = forward + backward."""

        def __init__(self, lin, tensors=None, seed=0, w_layout=0, max_sets=None):
            self.lin = lin
            lay = lin.layout
            # w_layout 2: the frozen weight is kept in both layouts and each direction gets the one whose contraction
            # index is contiguous (forward [d_out][d_in], backward [d_in][d_out])
            self.desc = gh.desc_of(lin, 1 if w_layout else 0)
            self.desc_bwd = gh.desc_of(lin, 1 if w_layout == 1 else 0)
            if tensors is None:
                x, W, dy, A, B = gpu_tensors(lin, seed)
            else:
                x, W, dy = (gh.to_dev(tensors.x, lin.dtype), gh.to_dev(tensors.W, lin.dtype), gh.to_dev(tensors.dy, lin.dtype))
                A = [gh.to_dev(a, lin.dtype) for a in tensors.A]
                B = [gh.to_dev(b, lin.dtype) for b in tensors.B]
            T, D, K = lay.T, lin.D, lin.K
            e = x.element_size()
            self.n_sets = max(1, -(-ROTATE_BYTES // max(min(T * D, T * K) * e, 1)))
            if max_sets:
                self.n_sets = min(self.n_sets, max_sets)
            self.xs = [x] + [x.clone() for _ in range(self.n_sets - 1)]
            self.dys = [dy] + [dy.clone() for _ in range(self.n_sets - 1)]
            self.W_bwd = W.t().contiguous() if w_layout == 1 else W      # [d_out][d_in] is the same matrix transposed in memory
            self.W = W.t().contiguous() if w_layout == 2 else self.W_bwd
            self.A, self.B = A, B
            self.y = torch.empty(T, K, dtype=x.dtype, device="cuda")
            self.dx = torch.empty(T, D, dtype=x.dtype, device="cuda")
            self.h = torch.empty(max(plora.plora_h_elems(self.desc), 1), dtype=torch.float32, device="cuda")
            self.dA = [torch.empty(D, int(r), dtype=torch.float32, device="cuda") for r in lay.rank]
            self.dB = [torch.empty(int(r), K, dtype=torch.float32, device="cuda") for r in lay.rank]
            self.ws = torch.empty(max(plora.plora_workspace_bytes(self.desc), plora.plora_workspace_bytes(self.desc_bwd)),
                                  dtype=torch.uint8, device="cuda")

        def fwd(self, i):
            plora.plora_linear_fwd(self.desc, self.xs[i % self.n_sets], self.W, self.A, self.B, self.y, self.h, self.ws)

        def bwd(self, i):
            plora.plora_linear_bwd(self.desc_bwd, self.xs[i % self.n_sets], self.W_bwd, self.A, self.B, self.dys[i % self.n_sets],
                                   self.h, self.dx, self.dA, self.dB, self.ws)

        def step(self, i):
            self.fwd(i)
            self.bwd(i)

    def work_of(lin):
        lay = lin.layout
        T, D, K = lay.T, lin.D, lin.K
        e = 2 if lin.dtype == "bf16" else 4
        sum_Lr = lay.sum_Lr()
        R = int(sum(int(r) for r in lay.rank))
        return {
            "gemm_fwd": ("mfma", 2.0 * T * D * K + 2.0 * K * sum_Lr),
            "gemm_dx": ("mfma", 2.0 * T * D * K + 2.0 * D * sum_Lr),
            "shrink": ("hbm", T * D * e + D * R * e + sum_Lr * 4.0),
            "dh": ("hbm", T * K * e + R * K * e + sum_Lr * 4.0),
            "db": ("hbm", T * K * e + sum_Lr * 4.0 + R * K * 4.0),
            "da": ("hbm", T * D * e + sum_Lr * 4.0 + D * R * 4.0),
        }

    def kernel_table(lin, kern_ms):
        out = {}
        for name, (bound, work) in work_of(lin).items():
            ms = kern_ms.get(name)
            if not ms:
                continue
            if bound == "mfma":
                a = work / (ms * 1e-3) / 1e12
                ent = {"ms": round(ms, 4), "bound": bound, "achieved": round(a, 1), "unit": "TFLOP/s",
                       "frac": round(a / PEAK_BF16_MFMA_TFLOPS, 4)}
                if ceil["mfma_only_tflops"]:
                    ent["frac_of_measured_ceiling"] = round(a / ceil["mfma_only_tflops"], 4)
            else:
                a = work / (ms * 1e-3) / 1e9
                ent = {"ms": round(ms, 4), "bound": bound, "achieved": round(a, 1), "unit": "GB/s",
                       "frac": round(a / PEAK_HBM_GBS, 4), "algorithmic_bytes": int(work)}
                if ceil["stream_read_gbs"]:
                    ent["frac_of_measured_ceiling"] = round(a / ceil["stream_read_gbs"], 4)
            out[name] = ent
        if kern_ms.get("prep"):
            out["prep"] = {"ms": round(kern_ms["prep"], 4)}
        return out

    def timed(step_fn, steps, warmup):
        for i in range(warmup):
            step_fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step_fn(warmup + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def graph_ms(step_fn, n_sets, reps=3):
        """The same steps recorded once in a HIP graph (one step per input set) and replayed: ms per step without the
        host's share of the launches."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step_fn(0)
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=side):
                for i in range(n_sets):
                    step_fn(i)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / (reps * n_sets)
        del g
        return ms

    def kernel_times(step_fn, steps):
        plora.plora_set_kernel_timing(True)
        for i in range(steps):
            step_fn(i)
        torch.cuda.synchronize()
        kern = {}
        for name in plora.KERNEL_CLASSES:
            if name in ("adamw", "expand", "nf4"):
                continue
            ms, n = plora.plora_kernel_time(name)
            kern[name] = (ms / n) if n else None
        plora.plora_set_kernel_timing(False)
        return kern

    def layer_steps(runs):
        """The seven linears of a decoder layer back to back, forward in order, backward in reverse: as seven plain
        calls each way, and with the projections that share an input (q / k / v on the layer's input, gate / up on the
        MLP's) as grouped calls.  The grouped calls use the first member's input sets as the shared x."""
        def plain(i):
            for r in runs:
                r.fwd(i)
            for r in reversed(runs):
                r.bwd(i)

        def group_of(idx):
            rs = [runs[j] for j in idx]
            g = plora.Group([r.desc for r in rs])
            return g, torch.empty(plora.plora_group_workspace_bytes(g), dtype=torch.uint8, device="cuda"), rs

        def gfwd(gr, i):
            g, ws, rs = gr
            plora.plora_group_fwd(g, rs[0].xs[i % rs[0].n_sets], [r.W for r in rs], [r.A for r in rs], [r.B for r in rs],
                                  [r.y for r in rs], [r.h for r in rs], ws)

        def gbwd(gr, i, summed=False):
            g, ws, rs = gr
            plora.plora_group_bwd(g, rs[0].xs[i % rs[0].n_sets], [r.W_bwd for r in rs], [r.A for r in rs], [r.B for r in rs],
                                  [r.dys[i % r.n_sets] for r in rs], [r.h for r in rs], None if summed else [r.dx for r in rs],
                                  [r.dA for r in rs], [r.dB for r in rs], ws, dx_sum=rs[0].dx if summed else None)

        if len(runs) != 7:
            return plain, None, None, None
        qkv, gate_up = group_of((0, 1, 2)), group_of((4, 5))

        def grouped(i):
            gfwd(qkv, i); runs[3].fwd(i); gfwd(gate_up, i); runs[6].fwd(i)
            runs[6].bwd(i); gbwd(gate_up, i); runs[3].bwd(i); gbwd(qkv, i)

        # the layer as a model runs it: the gradient of a shared input is the sum over the projections that read it.
        # Plain calls leave that to two elementwise additions for q / k / v and one for gate / up; the grouped calls
        # form it in the GEMM epilogues (dx_sum).
        def plain_summed(i):
            plain(i)
            torch.add(runs[4].dx, runs[5].dx, out=runs[4].dx)
            torch.add(runs[0].dx, runs[1].dx, out=runs[0].dx)
            torch.add(runs[0].dx, runs[2].dx, out=runs[0].dx)

        def grouped_summed(i):
            gfwd(qkv, i); runs[3].fwd(i); gfwd(gate_up, i); runs[6].fwd(i)
            runs[6].bwd(i); gbwd(gate_up, i, True); runs[3].bwd(i); gbwd(qkv, i, True)

        return plain, grouped, plain_summed, grouped_summed

    if args.linear < 0:
        # profiling mode: the linears of the configuration back to back (--grouped: q / k / v and gate / up as grouped calls)
        lins = wl.config(args.config)
        runs = [Runner(l, None, seed=1000 * args.config + i) for i, l in enumerate(lins)]
        plain_step, grouped_step, _, _ = layer_steps(runs)
        if args.grouped and grouped_step is None:
            raise SystemExit("--grouped needs the seven linears of configuration 4")
        layer_step = grouped_step if args.grouped else plain_step
        ms = timed(layer_step, args.steps, args.warmup)
        fl = sum(l.flops_fwd_bwd() for l in lins)
        print(json.dumps({"metric": "packed multi-LoRA layer fwd+bwd TFLOP/s", "value": round(fl / (ms * 1e-3) / 1e12, 2),
                          "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
                          "config": {"workload": f"config {args.config}: all {len(lins)} linears in sequence"
                                                 + (", q/k/v and gate/up as grouped calls" if args.grouped else "")}}))
        return

    # ---- headline workload ---------------------------------------------------------------------
    lin = wl.config(args.config)[args.linear]
    lay = lin.layout
    T, D, K = lay.T, lin.D, lin.K
    t = lin.tensors()
    w_layout = {"in_out": 0, "out_in": 1, "both": 2}[args.w_layout]
    run = Runner(lin, t, w_layout=w_layout)
    flops = lin.flops_fwd_bwd()

    if args.calib_copy:
        # known traffic for calibrating FETCH_SIZE / WRITE_SIZE: a 256 MiB device copy, and the two 1 GiB streaming
        # reads of the bench-side library (plain loads; direct-to-LDS loads, which is what the library's kernels use -
        # the counters weigh the two kinds of request differently)
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        blib_path = os.path.join(ROOT, "paper_2508_02932_amd", "libplora_bench.so")
        if os.path.exists(blib_path):
            bl = C.CDLL(blib_path)
            buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
            sink = torch.zeros(4, dtype=torch.float32, device="cuda")
            v = C.c_double(0)
            bl.plora_bench_stream_read(C.c_void_p(buf.data_ptr()), C.c_size_t(buf.numel()), 2, C.c_void_p(sink.data_ptr()),
                                       C.c_void_p(int(torch.cuda.current_stream().cuda_stream) or None), C.byref(v))
            del buf, sink

    ms_per_step = timed(run.step, args.steps, args.warmup)

    # spread of single steps (context; the metric above is the mean of the timed region): one event pair per step
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i, (a, b) in enumerate(evs):
        a.record()
        run.step(i)
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in evs)
    step_stats = {"median_ms": round(per_step[len(per_step) // 2], 4), "min_ms": round(per_step[0], 4),
                  "max_ms": round(per_step[-1], 4)}

    # host time of one call: the calls only enqueue, so timing them without synchronising measures the host side
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_host = 20
    for i in range(n_host):
        run.fwd(i)
    host_fwd_us = (time.perf_counter() - t0) * 1e6 / n_host
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n_host):
        run.bwd(i)
    host_bwd_us = (time.perf_counter() - t0) * 1e6 / n_host
    torch.cuda.synchronize()

    # second pass of the same steps with every kernel bracketed by HIP events on its stream
    kern = kernel_times(run.step, args.steps)
    kernels = kernel_table(lin, kern)

    # the per-adapter optimizer step that follows a backward call (not part of the step metric: the layer is the
    # forward and the backward call; reported as a kernel of its own against the HBM roofline)
    if lin.dtype == "bf16" and lay.n_adapters > 0:
        def side(params, grads):
            return {"param": params, "master": [p_.float() for p_ in params], "grad": grads,
                    "m": [torch.zeros_like(g_) for g_ in grads], "v": [torch.zeros_like(g_) for g_ in grads]}
        sA, sB = side(run.A, run.dA), side(run.B, run.dB)
        hps = [(2e-4, 0.9, 0.999, 1e-8, 0.01, 1)] * lay.n_adapters
        n_opt = 10
        for _ in range(2):
            plora.plora_adamw_step(run.desc, sA, sB, hps)
        torch.cuda.synchronize()
        plora.plora_set_kernel_timing(True)       # HIP events around the launches, on their stream
        for _ in range(n_opt):
            plora.plora_adamw_step(run.desc, sA, sB, hps)
        torch.cuda.synchronize()
        ms_tot, n_br = plora.plora_kernel_time("adamw")
        plora.plora_set_kernel_timing(False)
        ms_opt = ms_tot / max(n_br, 1)
        n_par = sum(int(r) for r in lay.rank) * (D + K)
        by = 30.0 * n_par                 # read master, g, m, v (16 B); write master, m, v (12 B) and the bf16 copy (2 B)
        a = by / (ms_opt * 1e-3) / 1e9
        kernels["adamw"] = {"ms": round(ms_opt, 4), "bound": "hbm", "achieved": round(a, 1), "unit": "GB/s",
                            "frac": round(a / PEAK_HBM_GBS, 4), "algorithmic_bytes": int(by), "parameters": n_par,
                            "note": "plora_adamw_step over all A_k, B_k (two launches); reads and writes, so the read-only "
                                    "streaming ceiling does not apply"}
        del sA, sB
        torch.cuda.empty_cache()

    # the stand-alone low-rank calls (for callers with a base GEMM of their own): y and dx are updated in place
    lora_only = None
    if lin.dtype == "bf16" and lay.n_adapters > 0:
        ws_lo = torch.empty(plora.plora_lora_workspace_bytes(run.desc), dtype=torch.uint8, device="cuda")
        n_lo = 10
        res = {}
        sum_Lr = lay.sum_Lr()
        R = int(sum(int(r) for r in lay.rank))
        rows = int(sum(int(lay.seg_off[s_ + 1] - lay.seg_off[s_]) for s_ in range(lay.n_seg) if int(lay.seg_adapter[s_]) >= 0))

        def lo_fwd(i):
            plora.plora_lora_fwd(run.desc, run.xs[i % run.n_sets], run.A, run.B, run.y, run.h, ws_lo)

        def lo_bwd(i):
            plora.plora_lora_bwd(run.desc, run.xs[i % run.n_sets], run.A, run.B, run.dys[i % run.n_sets], run.h, run.dx,
                                 run.dA, run.dB, ws_lo)

        for name, fn, N_ in (("fwd", lo_fwd, K), ("bwd", lo_bwd, D)):
            run.y.zero_()
            run.dx.zero_()
            ms_call = timed(fn, n_lo, 2)
            plora.plora_set_kernel_timing(True)
            for i in range(n_lo):
                fn(i)
            torch.cuda.synchronize()
            ms_tot, n_br = plora.plora_kernel_time("expand")
            plora.plora_set_kernel_timing(False)
            ms_k = ms_tot / max(n_br, 1)
            by = 2.0 * rows * N_ * 2 + sum_Lr * 2.0 + R * N_ * 2.0    # C read and written, low-rank factor, small matrices
            a = by / (ms_k * 1e-3) / 1e9
            res[name] = {"call_ms": round(ms_call, 4),
                         "expand_kernel": {"ms": round(ms_k, 4), "bound": "hbm", "achieved": round(a, 1), "unit": "GB/s",
                                           "frac": round(a / PEAK_HBM_GBS, 4), "algorithmic_bytes": int(by)}}
        res["note"] = ("plora_lora_fwd: shrink + in-place update of y; plora_lora_bwd: dH, dB, dA + in-place update of dx; "
                       "the update kernel reads and writes its output once")
        lora_only = res
        del ws_lo
        torch.cuda.empty_cache()

    # the same step on a base weight stored in 4 bits (NF4): every call first expands W into the workspace
    nf4_base = None
    if lin.dtype == "bf16" and (D * K) % 64 == 0 and w_layout != 2:
        codes_h, absmax_h = wl.nf4_storage(D * K, D, seed=args.config)
        codes_d, absmax_d = torch.from_numpy(codes_h).cuda(), torch.from_numpy(absmax_h).cuda()
        del codes_h, absmax_h
        ws_q = torch.empty(plora.plora_nf4_workspace_bytes(run.desc), dtype=torch.uint8, device="cuda")
        n_q = max(4, args.steps // 2)

        def q_step(i):
            plora.plora_linear_fwd_nf4(run.desc, run.xs[i % run.n_sets], codes_d, absmax_d, run.A, run.B, run.y, run.h, ws_q)
            plora.plora_linear_bwd_nf4(run.desc_bwd, run.xs[i % run.n_sets], codes_d, absmax_d, run.A, run.B,
                                       run.dys[i % run.n_sets], run.h, run.dx, run.dA, run.dB, ws_q)

        ms_q = timed(q_step, n_q, 2)
        plora.plora_set_kernel_timing(True)
        for i in range(n_q):
            q_step(i)
        torch.cuda.synchronize()
        ms_tot, n_br = plora.plora_kernel_time("nf4")
        plora.plora_set_kernel_timing(False)
        ms_k = ms_tot / max(n_br, 1)
        by = D * K * (0.5 + 4.0 / 64 + 2.0)      # indices and block constants read, bf16 values written
        a = by / (ms_k * 1e-3) / 1e9
        nf4_base = {"ms_per_step": round(ms_q, 4), "tflops": round(flops / (ms_q * 1e-3) / 1e12, 1),
                    "slowdown_vs_bf16_weight": round(ms_q / ms_per_step, 4),
                    "dequant_kernel": {"ms": round(ms_k, 4), "bound": "hbm", "achieved": round(a, 1), "unit": "GB/s",
                                       "frac": round(a / PEAK_HBM_GBS, 4), "algorithmic_bytes": int(by)},
                    "weight_bytes": {"nf4": int(D * K * (0.5 + 4.0 / 64)), "bf16": int(D * K * 2)},
                    "note": "plora_linear_fwd_nf4 + plora_linear_bwd_nf4 (two expansions per step); synthetic indices and "
                            "block constants; the stored weight is read as W" + ("[d_out][d_in]" if w_layout == 1 else "[d_in][d_out]")}
        del codes_d, absmax_d, ws_q
        torch.cuda.empty_cache()

    # context: the vendor GEMM library on the same operands (not part of the metric)
    vendor = None
    if not args.no_context and lin.dtype == "bf16":
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_v = 5
        out = {}
        W_io = run.W_bwd.t() if w_layout == 1 else run.W_bwd        # [d_in][d_out] (a view when only the other copy exists)
        for name, a_, b_, c_ in (("fwd", run.xs[0], W_io, run.y), ("dx", run.dys[0], W_io.t(), run.dx)):
            for _ in range(2):
                torch.matmul(a_, b_, out=c_)
            e0.record()
            for _ in range(n_v):
                torch.matmul(a_, b_, out=c_)
            e1.record()
            torch.cuda.synchronize()
            out[name + "_tflops"] = round(2.0 * T * D * K / (e0.elapsed_time(e1) / n_v * 1e-3) / 1e12, 1)
        vendor = dict(out, note="torch.matmul (hipBLASLt) on the same x, W, dy without the low-rank terms; context only")

    # context leg (not the metric): the same work issued one adapter at a time
    sequential = None
    if args.sequential and w_layout == 0 and lay.n_adapters > 0 and all(int(a) >= 0 for a in lay.seg_adapter) \
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
                           np.array([lay.scale[k]]), run.desc.dtype)
            assert plora.plora_workspace_bytes(d) <= run.ws.numel()
            n_h = L * int(lay.rank[k])
            subs.append((d, run.xs[0][lo:hi], run.y[lo:hi], run.dys[0][lo:hi], run.dx[lo:hi], [run.A[k]], [run.B[k]],
                         [run.dA[k]], [run.dB[k]], run.h[h_off:h_off + n_h]))
            h_off += n_h

        def seq_step(i):
            for d, x_, y_, dy_, dx_, A_, B_, dA_, dB_, h_ in subs:
                plora.plora_linear_fwd(d, x_, run.W, A_, B_, y_, h_, run.ws)
            for d, x_, y_, dy_, dx_, A_, B_, dA_, dB_, h_ in subs:
                plora.plora_linear_bwd(d, x_, run.W, A_, B_, dy_, h_, dx_, dA_, dB_, run.ws)

        n_seq = max(3, args.steps // 4)
        seq_ms = timed(seq_step, n_seq, 2)
        sequential = {"ms_per_step": round(seq_ms, 4), "steps": n_seq, "calls_per_step": 2 * len(subs),
                      "packed_speedup": round(seq_ms / ms_per_step, 3),
                      "note": "same library, one forward and one backward call per adapter on its own rows"}

    # ---- fabric traffic of the dominant kernel: committed rocprofv3 summary of this very workload, used only
    # if it was taken from the kernel source as it stands now (otherwise null)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{lin.name}.txt")
    if os.path.exists(tpath):
        import hashlib
        src = os.path.join(ROOT, "paper_2508_02932_amd", "csrc", "gemm_bf16.hip")
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
        vals = {}
        for line in open(tpath):
            parts = line.split()
            if len(parts) >= 2 and not line.startswith("#"):
                vals[parts[0]] = parts[1]
        if vals.get("kernel_source_sha16") == sha and "gemm_fwd" in vals:
            traffic = float(vals["gemm_fwd"])
    dom = kernels.get("gemm_fwd", {})
    roofline = {"kernel": "k_gemm<forward> (x W with fused scale*h*B_k)", "bound": "mfma",
                "achieved": dom.get("achieved"), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": dom.get("frac"), "traffic": traffic, "avg_launch_ms": dom.get("ms"),
                "frac_of_measured_ceiling": dom.get("frac_of_measured_ceiling")}
    rotation = {"input_sets": run.n_sets, "bytes_of_x_and_dy_per_set": int(T * (D + K) * 2),
                "note": "x and dy of step i come from set i mod input_sets; the sets of one tensor total more than "
                        f"{ROTATE_BYTES >> 20} MB"}

    # ---- the other configurations -----------------------------------------------------------------
    per_config = None
    layer_cost = None
    if not args.no_per_config:
        headline = (args.config, args.linear)
        del run
        torch.cuda.empty_cache()
        per_config = []
        n_pc = max(4, args.steps // 2)
        for cfg in (2, 3, 4, 5):
            lins = wl.config(cfg)
            entries = []
            for li, l2 in enumerate(lins):
                if (cfg, li) == headline:
                    continue
                if cfg == 5 and li == 1:
                    continue                      # the 28672-wide linear is the default headline; skip unless chosen
                r2 = Runner(l2, None, seed=1000 * cfg + li)
                ms2 = timed(r2.step, n_pc, 3)
                k2 = kernel_times(r2.step, n_pc)
                f2 = l2.flops_fwd_bwd()
                entries.append((l2, r2, {"workload": f"config {cfg} / {l2.name}: d_in={l2.D} d_out={l2.K} T={l2.layout.T} "
                                                     f"adapters={l2.layout.n_adapters}",
                                         "ms_per_step": round(ms2, 4), "tflops": round(f2 / (ms2 * 1e-3) / 1e12, 1),
                                         "tokens_per_s": round(l2.layout.T / (ms2 * 1e-3), 1), "input_sets": r2.n_sets,
                                         "graph_replay_ms_per_step": round(graph_ms(r2.step, r2.n_sets), 4),
                                         "kernels": kernel_table(l2, k2)}))
                if cfg != 4:
                    del r2
                    entries[-1] = (l2, None, entries[-1][2])
                    torch.cuda.empty_cache()
            if cfg == 4:
                runs = [r for _, r, _ in entries]
                layer_step, grouped_step, plain_summed, grouped_summed = layer_steps(runs)
                ms4 = timed(layer_step, n_pc, 3)
                ms4g = timed(grouped_step, n_pc, 3)
                ms4ps = timed(plain_summed, n_pc, 3)
                ms4gs = timed(grouped_summed, n_pc, 3)
                # the same layer on one configuration's own small batch (512 tokens, one adapter): with the full batch it
                # gives the planner's cost model, time(tokens) = floor + slope * tokens
                small_T = 512
                small_runs = [Runner(wl.Linear(l.name + "_small", "bf16", l.D, l.K, wl.equal_layout(1, small_T, [16], [2.0]), 0.02,
                                               wl.BASE_SEED + 4900 + j), None, seed=4900 + j, max_sets=8) for j, (l, _, _) in enumerate(entries)]
                ms4s = timed(layer_steps(small_runs)[1], 4 * n_pc, 5)
                del small_runs
                slope = (ms4g - ms4s) / (entries[0][0].layout.T - small_T)
                layer_cost = {"floor_ms": ms4s - slope * small_T, "ms_per_token": slope, "small_batch_tokens": small_T,
                              "small_batch_ms": ms4s, "full_batch_tokens": entries[0][0].layout.T, "full_batch_ms": ms4g}
                kp, kg = kernel_times(layer_step, n_pc), kernel_times(grouped_step, n_pc)
                f4 = sum(l.flops_fwd_bwd() for l, _, _ in entries)
                per_config.append({"workload": "config 4: the seven linears of a decoder layer (q,k,v,o,gate,up,down), forward "
                                               "in order then backward in reverse, one stream",
                                   "ms_per_step": round(ms4, 4), "tflops": round(f4 / (ms4 * 1e-3) / 1e12, 1),
                                   "tokens_per_s": round(entries[0][0].layout.T / (ms4 * 1e-3), 1),
                                   "graph_replay_ms_per_step": round(graph_ms(layer_step, min(r.n_sets for r in runs)), 4),
                                   "grouped": {"ms_per_step": round(ms4g, 4), "tflops": round(f4 / (ms4g * 1e-3) / 1e12, 1),
                                               "graph_replay_ms_per_step": round(graph_ms(grouped_step, min(r.n_sets for r in runs)), 4),
                                               "ms_per_step_in_kernel": {k: {"plain_7_launches": round(7 * kp[k], 4),
                                                                             "grouped_4_launches": round(4 * kg[k], 4)}
                                                                         for k in ("shrink", "da") if kp.get(k) and kg.get(k)},
                                               "with_input_gradients_summed": {
                                                   "plain_calls_plus_three_additions_ms": round(ms4ps, 4),
                                                   "grouped_dx_sum_ms": round(ms4gs, 4),
                                                   "note": "the gradient of a shared input is the sum over the projections that read "
                                                           "it: plain calls plus torch.add (two for q/k/v, one for gate/up) against "
                                                           "the grouped calls' dx_sum (summed in the GEMM epilogues)"},
                                               "note": "plora_group_fwd / _bwd for q,k,v (one x) and gate,up (one x): one "
                                                       "shrink pass and one dA pass over x per group; o and down as plain calls"},
                                   "linears": [e for _, _, e in entries]})
                del runs
                for i in range(len(entries)):
                    entries[i] = (entries[i][0], None, entries[i][2])
                torch.cuda.empty_cache()
            else:
                per_config += [e for _, _, e in entries]
        # the headline linear with the frozen weight stored the other way round (the forward and backward GEMMs
        # swap forms: the one that contracts over W's contiguous index runs forward)
        if lin.dtype == "bf16":
            names = {0: "[d_in][d_out]", 1: "[d_out][d_in]",
                     2: "in both layouts (frozen, so one extra copy in HBM buys each direction the GEMM form that "
                        "contracts over W's contiguous index)"}
            for other in (0, 1, 2):
                if other == w_layout:
                    continue
                r3 = Runner(lin, t, w_layout=other)
                ms3 = timed(r3.step, n_pc, 3)
                k3 = kernel_times(r3.step, n_pc)
                per_config.append({"workload": f"config {args.config} / {lin.name} with W stored " + names[other],
                                   "ms_per_step": round(ms3, 4), "tflops": round(flops / (ms3 * 1e-3) / 1e12, 1),
                                   "tokens_per_s": round(T / (ms3 * 1e-3), 1), "input_sets": r3.n_sets,
                                   "kernels": kernel_table(lin, k3)})
                del r3
                torch.cuda.empty_cache()

    # ---- CPU baseline: the oracle on a bounded sample of the headline workload -------------------------
    cpu = None
    if not args.no_cpu:
        import oracle
        from util import make_problem
        p = make_problem(oracle, lin, t)
        rng = np.random.default_rng(0)
        cores = oracle.loops.threads()
        sum_Lr = lay.sum_Lr()

        def rows_time(n):
            rows = np.sort(rng.choice(T, size=min(n, T), replace=False))
            a = time.perf_counter()
            oracle.loops.fwd_rows(p, rows)
            oracle.loops.bwd_rows(p, t.dy, rows)
            return time.perf_counter() - a, len(rows)

        probe_s, probe_n = rows_time(2 * cores)
        n_rows = int(max(2 * cores, min(T, 10.0 / max(probe_s / probe_n, 1e-6))))
        rows_s, n_rows = rows_time(n_rows)
        # weight gradients: every adapter when that stays within a few seconds, else the largest-rank one
        k_big = int(np.argmax(lay.rank))
        Lr = [sum(int(lay.seg_off[s + 1] - lay.seg_off[s]) * int(lay.rank[k])
                  for s in range(lay.n_seg) if lay.seg_adapter[s] == k) for k in range(lay.n_adapters)]
        a = time.perf_counter()
        oracle.loops.grad_adapter(p, t.dy, k_big)
        one_s = time.perf_counter() - a
        done = [k_big]
        if one_s * (sum_Lr / max(Lr[k_big], 1)) < 12.0:
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
                         + ("the whole step, nothing extrapolated" if whole else
                            "whole step extrapolated: row part scaled by T / rows, weight gradients by sum(L r)")}

    # context leg (host only, not the metric): the packing planner on a search space of the paper's size, its cost
    # model filled from the decoder-layer times measured above
    planner = None
    if layer_cost is not None:
        rng = np.random.default_rng(120)
        n_cfg, n_gpus_plan, n_layers, iters, seq = 120, 8, 32, 1000, 512
        ranks = rng.choice([8, 16, 32, 64, 128], n_cfg)
        batch = rng.choice([1, 2, 4, 8], n_cfg)
        tokens = batch * seq
        model = dict(n_layers=n_layers, hidden=4096, kv_hidden=1024, inter=14336, c_prec=2.0, c_grad=3.0)
        mem = np.array([plora.plora_plan_lora_bytes(model, dict(rank=int(r), batch=int(b_), seq=seq, targets=127))
                        for r, b_ in zip(ranks, batch)])
        # the base model's activations kept for the backward pass grow with the packed tokens as well: charged to the configuration
        mem = mem + tokens * (4096 * 16 + 14336 * 3) * 2.0 * n_layers
        per_iter = n_layers * 1e-3                                          # ms of one layer -> seconds of all layers
        eff = [2 ** i * 0.9 ** i for i in range(4)]                          # assumed speed-up of 2^i GPUs (one GPU here)
        t_base = [60.0 + iters * per_iter * max(layer_cost["floor_ms"], 0.0) / e for e in eff]
        t_cfg = np.array([iters * per_iter * layer_cost["ms_per_token"] * tokens / e for e in eff])
        prob = plora.PlanProblem(ranks, mem, 16.1e9, 288.0e9, 0.9, t_base, t_cfg)
        t0p = time.perf_counter()
        sched = plora.plora_plan_schedule(prob, n_gpus_plan)
        plan_ms = (time.perf_counter() - t0p) * 1e3
        alone = float(sum(t_base[0] + t_cfg[0][k] for k in range(n_cfg))) / n_gpus_plan
        all_gpus = float(sum(t_base[3] + t_cfg[3][k] for k in range(n_cfg)))      # one configuration at a time on all 8 GPUs
        planner = {"configs": n_cfg, "gpus": n_gpus_plan, "planning_ms": round(plan_ms, 2), "jobs": len(sched["jobs"]),
                   "makespan_s": round(sched["makespan"], 1), "work_over_gpus_s": round(sched["gpu_work"] / n_gpus_plan, 1),
                   "tail_bound": round(sched["tail_bound"], 4), "all_packings_proved_optimal": sched["all_proved"],
                   "one_configuration_per_job_s": round(alone, 1),
                   "speedup_over_one_configuration_per_job": round(alone / sched["makespan"], 3),
                   "one_configuration_on_all_gpus_s": round(all_gpus, 1),
                   "layer_cost_model": {k: round(v, 6) for k, v in layer_cost.items()},
                   "note": "plora_plan_schedule (DTM + job planner) on 120 synthetic configurations (ranks 8-128, batches of 1-8 "
                           "sequences of 512 tokens, 1000 iterations, 8B-shaped model of 32 layers, 8 GPUs of 288 GB).  Cost model: "
                           "iteration = 32 x (floor + slope x packed tokens) from the two decoder-layer timings above, 60 s per job "
                           "to load the model, parallel speed-up 1.8 per doubling ASSUMED (one GPU here); memory from the appendix-B "
                           "model plus the base activations of the packed tokens.  one_configuration_per_job_s: the same 120 "
                           "runs unpacked, one GPU each, spread evenly over the 8 GPUs (the paper's Min GPU baseline); "
                           "one_configuration_on_all_gpus_s: one after the other on all 8 (its Max GPU baseline)"}

    out = {
        "metric": "packed multi-LoRA layer fwd+bwd TFLOP/s",
        "value": round(flops / (ms_per_step * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s",
        "tokens_per_s": round(T / (ms_per_step * 1e-3), 1),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "step_ms": step_stats,
        "host_us_per_call": {"fwd": round(host_fwd_us, 1), "bwd": round(host_bwd_us, 1)},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if lin.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"config {args.config} / {lin.name}: d_in={D} d_out={K} T={T} "
                               f"adapters={lay.n_adapters} ranks={sorted(set(int(r) for r in lay.rank))}"
                               + ("", " W stored [d_out][d_in]", " W stored in both layouts")[w_layout],
                   "tokens": T, "d_in": D, "d_out": K, "n_adapters": lay.n_adapters,
                   "flops_per_step": flops},
        "frac_of_bf16_mfma_peak": round(flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4),
        "roofline": roofline,
        "kernels": kernels,
        "measured_ceilings": ceil,
        "rotation": rotation,
        "lora_only": lora_only,
        "nf4_base": nf4_base,
        "vendor_gemm": vendor,
        "sequential_adapters": sequential,
        "per_config": per_config,
        "planner": planner,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
