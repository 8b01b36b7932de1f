"""GPU parity of the per-adapter AdamW step (plora_adamw_step) against the fp64 oracle
(oracle/adamw.py), element by element, over several steps with different hyperparameters per
adapter.  fp32 arithmetic against fp64: the scaled error bound is 1e-6 (a handful of roundings of
2^-24 each per step; a wrong term of the rule shows up at 1e-3 or more).  The bf16 copy of the
parameters is a rounding decision: it must equal the fp32 master copy rounded to nearest even, bit
for bit."""
import numpy as np
import pytest

import oracle
from oracle.adamw import Hyper
from paper_2508_02932_amd import workloads as wl
from util import scaled_err

pytestmark = pytest.mark.gpu
TOL = 1e-6


def f32(x) -> float:
    """The value an fp32 argument of the C interface carries (both sides get the same hyperparameters)."""
    return float(np.float32(x))


def run_steps(dtype, D, K, ranks, hps, n_steps, with_master=True, seed=0):
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    rng = np.random.default_rng(seed)
    n = len(ranks)
    lin = wl.small(f"adamw_{dtype}", dtype, D, K, lengths=[8] * n, seg_adapter=list(range(n)), ranks=ranks,
                   scales=[1.0] * n, seed=seed)
    t = lin.tensors(want=("A", "B"))
    desc = gh.desc_of(lin)
    shapes = {"A": [(D, r) for r in ranks], "B": [(r, K) for r in ranks]}
    host = {"A": [a.astype(np.float64) for a in t.A], "B": [b.astype(np.float64) for b in t.B]}
    state = {s: {"m": [rng.standard_normal(sh) * 0.01 if k == 1 else np.zeros(sh) for k, sh in enumerate(shapes[s])],
                 "v": [np.abs(rng.standard_normal(sh)) * 1e-3 if k == 1 else np.zeros(sh) for k, sh in enumerate(shapes[s])]}
             for s in "AB"}
    g = []
    dev = {}
    for s in "AB":
        src = t.A if s == "A" else t.B
        dev[s] = {"param": [gh.to_dev(a, dtype) for a in src],
                  "master": [torch.from_numpy(a.astype(np.float32)).cuda() for a in src] if with_master else None,
                  "m": [torch.from_numpy(m.astype(np.float32)).cuda() for m in state[s]["m"]],
                  "v": [torch.from_numpy(v.astype(np.float32)).cuda() for v in state[s]["v"]]}
        # the oracle starts from the fp32 values the device holds
        state[s]["m"] = [m.astype(np.float32).astype(np.float64) for m in state[s]["m"]]
        state[s]["v"] = [v.astype(np.float32).astype(np.float64) for v in state[s]["v"]]
    for step in range(n_steps):
        print(f"[case] adamw {dtype} step {step + 1} ranks={ranks} master={with_master}", flush=True)
        grads = {s: [(rng.standard_normal(sh) * 0.05).astype(np.float32) for sh in shapes[s]] for s in "AB"}
        hp_now = [Hyper(f32(h.lr), f32(h.beta1), f32(h.beta2), f32(h.eps), f32(h.weight_decay), h.step + step, f32(h.grad_scale))
                  for h in hps]
        for s in "AB":
            dev[s]["grad"] = [torch.from_numpy(gr).cuda() for gr in grads[s]]
        plora.plora_adamw_step(desc, dev["A"], dev["B"],
                               [(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, h.step, h.grad_scale) for h in hp_now])
        torch.cuda.synchronize()
        A2, B2, mA, vA, mB, vB = oracle.adamw.step_adapters(host["A"], host["B"], grads["A"], grads["B"], state["A"]["m"],
                                                            state["A"]["v"], state["B"]["m"], state["B"]["v"], hp_now)
        host["A"], host["B"] = A2, B2
        state["A"]["m"], state["A"]["v"], state["B"]["m"], state["B"]["v"] = mA, vA, mB, vB
        errs = {}
        for s in "AB":
            for k in range(n):
                th = dev[s]["master"][k] if with_master else dev[s]["param"][k]
                errs[f"{s}{k}"] = scaled_err(gh.to_np(th), host[s][k])
                errs[f"m{s}{k}"] = scaled_err(gh.to_np(dev[s]["m"][k]), state[s]["m"][k])
                errs[f"v{s}{k}"] = scaled_err(gh.to_np(dev[s]["v"][k]), state[s]["v"][k])
                if with_master:
                    want = gh.to_np(dev[s]["master"][k])
                    if dtype == "bf16":
                        want = wl.round_to_bf16(want)
                    assert np.array_equal(gh.to_np(dev[s]["param"][k]), want), (s, k)
        worst = max(errs.values())
        print(f"  worst scaled error {worst:.2e}", flush=True)
        assert all(np.isfinite(v) and v <= TOL for v in errs.values()), {k: v for k, v in errs.items() if not v <= TOL}


HP3 = [Hyper(2e-3, 0.9, 0.999, 1e-8, 0.0, 1), Hyper(4e-4, 0.8, 0.95, 1e-6, 0.1, 5, 0.125), Hyper(2e-5, 0.9, 0.99, 1e-8, 0.01, 1, 3.0)]


def test_adamw_bf16_three_adapters_three_steps():
    run_steps("bf16", 264, 136, [8, 33, 128], HP3, 3)


def test_adamw_f32_in_place_and_with_master():
    run_steps("f32", 10, 14, [1, 3, 5], HP3, 2, with_master=False)      # tensor sizes that are no multiple of 4
    run_steps("f32", 64, 40, [4, 8, 2], HP3, 2, with_master=True)


def test_adamw_more_tensors_than_one_launch_carries():
    n = 25                                                               # 50 tensors: two launches
    hps = [Hyper(1e-3 * (1 + k % 3), 0.9, 0.99, 1e-8, 0.02 * (k % 2), 1 + k % 4, (1.0, 0.5, 1.0 / 1024)[k % 3]) for k in range(n)]
    run_steps("bf16", 72, 56, [1 + (7 * k) % 24 for k in range(n)], hps, 2)


def test_adamw_at_the_size_of_configuration_5():
    """All 64 adapter matrices of the largest linear (8192 -> 28672, 32 adapters, 41.6 M parameters): the launch
    configuration bench.py times, every element against the oracle."""
    lay = wl.config(5)[1].layout
    ranks = [int(r) for r in lay.rank]
    hps = [Hyper(1e-4 * (1 + k % 5), 0.9, 0.999 if k % 2 else 0.95, 1e-8, 0.01 * (k % 3), 1 + k % 7) for k in range(len(ranks))]
    run_steps("bf16", 8192, 28672, ranks, hps, 1, seed=5)


def test_adamw_rejects_bad_arguments():
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    lin = wl.small("adamw_bad", "bf16", 16, 16, lengths=[4], seg_adapter=[0], ranks=[4], scales=[1.0])
    d = gh.desc_of(lin)
    z = lambda *sh: [torch.zeros(*sh, device="cuda")]
    side = lambda: {"param": [torch.zeros(16, 4, device="cuda", dtype=torch.bfloat16)], "master": z(16, 4), "grad": z(16, 4),
                    "m": z(16, 4), "v": z(16, 4)}
    ok = (1e-3, 0.9, 0.99, 1e-8, 0.0, 1)
    plora.plora_adamw_step(d, side(), side(), [ok])
    for bad, code in (((1e-3, 0.9, 0.99, 1e-8, 0.0, 0), 2), ((1e-3, 1.0, 0.99, 1e-8, 0.0, 1), 2),
                      ((1e-3, 0.9, 0.99, 1e-8, 0.0, 1, float("inf")), 2)):
        with pytest.raises(plora.PloraError) as e:
            plora.plora_adamw_step(d, side(), side(), [bad])
        assert e.value.code == code
    no_master = side()
    no_master["master"] = None
    with pytest.raises(plora.PloraError) as e:                           # bf16 needs the fp32 master copy
        plora.plora_adamw_step(d, no_master, side(), [ok])
    assert e.value.code == 1
    torch.cuda.synchronize()
