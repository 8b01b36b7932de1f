"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration
bench.py times.

Config 1 and 2: every element of every output against the oracle (config 1 in test_gpu_parity).
Configs 3-5: the outputs the scalar-loop oracle can compute one by one - rows of y, h and dx around
every segment boundary, around GEMM tile boundaries and at random positions; dA_k and dB_k in full
for the adapters of smallest and largest rank and one more - plus adjoint identities that hold at
any size and involve every element:
    <dy, f(u)> = <dx, u>            f linear in x           (dx from backward with the same dy)
    <dy, f_W=0(A := U)> = sum_k <dA_k, U_k>                 (dA_k does not depend on A_k)
    <dy, f_W=0(B := V)> = sum_k <dB_k, V_k>                 (dB_k does not depend on B_k)
"""
import sys
import time

import numpy as np
import pytest

import oracle
from paper_2508_02932_amd import workloads as wl
from util import make_problem, scaled_err

pytestmark = pytest.mark.gpu
TOL = 2e-2


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def sample_rows(lay, rng, n_random=32, max_rows=160):
    T = lay.T
    rows = {0, T - 1}
    for b in lay.seg_off[1:-1]:
        rows.update(int(b) + d for d in (-2, -1, 0, 1))
    for b in range(256, T, 256):
        if rng.random() < 0.15:
            rows.update((b - 1, b))
    rows = sorted(r for r in rows if 0 <= r < T)
    if len(rows) > max_rows - n_random:
        keep = rng.choice(len(rows), size=max_rows - n_random, replace=False)
        rows = sorted(rows[i] for i in keep)
    rows = sorted(set(rows) | set(int(v) for v in rng.integers(0, T, size=n_random)))
    return np.array(rows, dtype=np.int64)


def test_config2_full_tensors():
    import torch
    import gpu_harness as gh
    lin = wl.config(2)[0]
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    say(f"[case] {lin.name} full tensors vs matmul oracle")
    y_o, h_o = oracle.matmul.forward(p)
    dx_o, g_o, dA_o, dB_o = oracle.matmul.backward(p, t.dy)
    dp = gh.upload(lin, t)
    gh.forward(dp)
    gh.backward(dp)
    torch.cuda.synchronize()
    errs = {"y": scaled_err(gh.to_np(dp.y), y_o), "dx": scaled_err(gh.to_np(dp.dx), dx_o),
            "h": scaled_err(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)), h_o)}
    for k in range(lin.layout.n_adapters):
        errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o[k])
        errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o[k])
    say("  errors " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    assert all(np.isfinite(v) and v <= TOL for v in errs.values()), errs
    # the scalar-loop oracle on a few rows, as a cross-check of the matmul writing at this size
    rows = np.array([0, 2047, 2048, 4095, 4096, 8191])
    ys, _ = oracle.loops.fwd_rows(p, rows)
    assert scaled_err(ys, y_o[rows]) < 1e-12


def inner(a, b):
    import torch
    return float((a.double() * b.double()).sum().item())


def check_sampled_and_adjoint(lin):
    import torch
    import gpu_harness as gh
    rng = np.random.default_rng(1234)
    lay = lin.layout
    t0 = time.time()
    t = lin.tensors()
    say(f"[case] {lin.name} T={lay.T} D={lin.D} K={lin.K} ranks={lay.rank.tolist()} (inputs drawn in {time.time() - t0:.1f} s)")
    p = make_problem(oracle, lin, t)
    dp = gh.upload(lin, t)
    say("  forward")
    gh.forward(dp)
    torch.cuda.synchronize()
    say("  backward")
    gh.backward(dp)
    torch.cuda.synchronize()

    rows = sample_rows(lay, rng)
    t0 = time.time()
    y_o, h_o = oracle.loops.fwd_rows(p, rows)
    dx_o, _ = oracle.loops.bwd_rows(p, t.dy, rows)
    say(f"  oracle: {len(rows)} rows in {time.time() - t0:.1f} s")
    idx = torch.from_numpy(rows).cuda()
    errs = {"y": scaled_err(gh.to_np(dp.y[idx]), y_o), "dx": scaled_err(gh.to_np(dp.dx[idx]), dx_o)}
    h_rows = gh.ragged_h_to_rows(lin, gh.to_np(dp.h))[rows]
    errs["h"] = scaled_err(h_rows, h_o)
    ks = sorted({int(np.argmin(lay.rank)), int(np.argmax(lay.rank)), int(rng.integers(lay.n_adapters))})
    t0 = time.time()
    for k in ks:
        dA_o, dB_o = oracle.loops.grad_adapter(p, t.dy, k)
        errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o)
        errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o)
    say(f"  oracle: dA, dB of adapters {ks} in {time.time() - t0:.1f} s")
    say("  errors " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    assert all(np.isfinite(v) and v <= TOL for v in errs.values()), errs

    # ---- adjoint identities over all elements (bf16 outputs: agreement to a few 1e-3 of the norms)
    def rel(a, b, scale):
        return abs(a - b) / scale

    gen = torch.Generator(device="cuda").manual_seed(7)
    u = torch.randn(dp.x.shape, device="cuda", generator=gen).to(torch.bfloat16)
    y_u = torch.empty_like(dp.y)
    say("  adjoint in x")
    from paper_2508_02932_amd import plora
    plora.plora_linear_fwd(dp.desc, u, dp.W, dp.A, dp.B, y_u, None, dp.ws)
    torch.cuda.synchronize()
    lhs, rhs = inner(dp.dy, y_u), inner(dp.dx, u)
    scale = float(dp.dy.double().norm().item() * y_u.double().norm().item())
    say(f"    <dy,f(u)>={lhs:.6e} <dx,u>={rhs:.6e} rel={rel(lhs, rhs, scale):.2e}")
    assert rel(lhs, rhs, scale) < 2e-3
    del u

    W0 = torch.zeros_like(dp.W)
    say("  adjoint in A")
    U = [torch.randn(a.shape, device="cuda", generator=gen).to(torch.bfloat16) * (1.0 / 64) for a in dp.A]
    plora.plora_linear_fwd(dp.desc, dp.x, W0, U, dp.B, y_u, None, dp.ws)
    torch.cuda.synchronize()
    lhs = inner(dp.dy, y_u)
    rhs = sum(inner(dA, Uk) for dA, Uk in zip(dp.dA, U))
    scale = float(dp.dy.double().norm().item() * y_u.double().norm().item())
    say(f"    lhs={lhs:.6e} rhs={rhs:.6e} rel={rel(lhs, rhs, scale):.2e}")
    assert rel(lhs, rhs, scale) < 2e-3
    say("  adjoint in B")
    V = [torch.randn(b.shape, device="cuda", generator=gen).to(torch.bfloat16) * 0.125 for b in dp.B]
    plora.plora_linear_fwd(dp.desc, dp.x, W0, dp.A, V, y_u, None, dp.ws)
    torch.cuda.synchronize()
    lhs = inner(dp.dy, y_u)
    rhs = sum(inner(dB, Vk) for dB, Vk in zip(dp.dB, V))
    scale = float(dp.dy.double().norm().item() * y_u.double().norm().item())
    say(f"    lhs={lhs:.6e} rhs={rhs:.6e} rel={rel(lhs, rhs, scale):.2e}")
    assert rel(lhs, rhs, scale) < 2e-3


@pytest.mark.parametrize("which", [0, 1], ids=["mlp_up", "mlp_down"])
def test_config3_sampled(which):
    check_sampled_and_adjoint(wl.config(3)[which])


@pytest.mark.parametrize("which", range(7), ids=["q", "k", "v", "o", "gate", "up", "down"])
def test_config4_sampled(which):
    check_sampled_and_adjoint(wl.config(4)[which])


@pytest.mark.parametrize("which", [0, 1], ids=["attn", "mlp_up"])
def test_config5_sampled(which):
    check_sampled_and_adjoint(wl.config(5)[which])


def test_odd_shapes_many_tiles():
    """More GEMM tiles than workgroups of the persistent grid (18 x 18 of them, a count that the XCD
    remap does not divide), ragged in every dimension: rows, columns and contraction length are no
    multiples of the tile, segments of unequal length with a base-only one and an adapter that owns
    two segments, ranks from 1 to 128.  The narrow hidden sizes also send dA and dB through the
    128-column tiles with a split token walk."""
    lin = wl.small("odd_many_tiles", "bf16", 1096, 4360,
                   lengths=[611, 1290, 3, 0, 977, 258, 1031, 307],
                   seg_adapter=[0, 1, 2, 3, -1, 4, 1, 5],
                   ranks=[128, 1, 24, 8, 72, 33], scales=[2.0, 0.5, 1.0, 4.0, 2.0, 0.25], seed=83)
    assert ((lin.layout.T + 255) // 256) * ((lin.K + 255) // 256) > 256
    check_sampled_and_adjoint(lin)
    # and with the roles of the hidden sizes swapped (wide contraction, narrow output)
    lin = wl.small("odd_many_tiles_T", "bf16", 4360, 1096,
                   lengths=[611, 1290, 3, 0, 977, 258, 1031, 307],
                   seg_adapter=[0, 1, 2, 3, -1, 4, 1, 5],
                   ranks=[128, 1, 24, 8, 72, 33], scales=[2.0, 0.5, 1.0, 4.0, 2.0, 0.25], seed=89)
    check_sampled_and_adjoint(lin)
