"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration
bench.py times.

Config 1 and 2: every element of every output against the oracle (config 1 in test_gpu_parity).
Configs 3-5 and the odd-shaped cases, per linear:
  * h (the saved activation x A_k), dA_k and dB_k of EVERY adapter: every element against the
    matmul writing of the oracle (section 2.4; appendix C.2 cases 1-3);
  * y and dx: whole 256-row tiles spread over the batch (16 of them = 4096 rows, first and last tile
    included), the rows around every segment boundary and around the boundaries of the first and
    last tile of every segment, and seeded random rows - every element of those rows against the
    oracle (appendix C.2 case 4 for dx);
  * every other row of y and dx: the row-wise adjoint identity <dy_t, f(u)_t> = <dx_t, u_t>, held
    to the rounding noise of that row (tests/fullsize_checks.py; its power is shown by the CPU
    mutation tests in tests/test_fullsize_checks.py);
  * guard bands around every output and the workspace.
"""
import sys
import time

import numpy as np
import pytest

import oracle
import fullsize_checks as fc
from paper_2508_02932_amd import workloads as wl
from util import make_problem, scaled_err

pytestmark = pytest.mark.gpu
TOL = 2e-2


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


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
    gh.check_guards(dp)
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


def check_full_size(lin, n_whole_tiles=16, n_random=256, w_layout=0):
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    rng = np.random.default_rng(1234)
    lay = lin.layout
    t0 = time.time()
    t = lin.tensors()
    say(f"[case] {lin.name} T={lay.T} D={lin.D} K={lin.K} ranks={lay.rank.tolist()} w_layout={w_layout} "
        f"(inputs drawn in {time.time() - t0:.1f} s)")
    p = make_problem(oracle, lin, t)
    dp = gh.upload(lin, t, w_layout)
    say("  forward")
    gh.forward(dp)
    torch.cuda.synchronize()
    say("  backward")
    gh.backward(dp)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    errs = {}

    # ---- every element of h, dA_k, dB_k
    t0 = time.time()
    h_o = oracle.matmul.low_rank_activation(p)
    dA_o, dB_o = oracle.matmul.low_rank_gradients(p, t.dy)
    say(f"  oracle: h, dA, dB of all {lay.n_adapters} adapters in {time.time() - t0:.1f} s")
    errs["h"] = fc.compare(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)), h_o)
    for k in range(lay.n_adapters):
        errs[f"dA{k}"] = fc.compare(gh.to_np(dp.dA[k]), dA_o[k])
        errs[f"dB{k}"] = fc.compare(gh.to_np(dp.dB[k]), dB_o[k])
    del h_o, dA_o, dB_o

    # ---- row blocks of y and dx
    rows = fc.plan_rows(lay.seg_off, n_whole_tiles, n_random, rng)
    t0 = time.time()
    sub = p.take_rows(rows)
    y_o, _ = oracle.matmul.forward(sub)
    dx_o, _, _, _ = oracle.matmul.backward(sub, t.dy[rows])
    say(f"  oracle: y, dx of {len(rows)} rows in {time.time() - t0:.1f} s")
    idx = torch.from_numpy(rows).cuda()
    errs["y"] = fc.compare(gh.to_np(dp.y[idx]), y_o)
    errs["dx"] = fc.compare(gh.to_np(dp.dx[idx]), dx_o)
    del y_o, dx_o, sub
    worst = max(errs.values())
    say("  errors " + " ".join(f"{k}={v:.2e}" for k, v in errs.items() if k in ("h", "y", "dx") or v == worst)
        + f" (max over {len(errs)} tensors {worst:.2e})")
    assert all(np.isfinite(v) and v <= TOL for v in errs.values()), errs

    # ---- every row: <dy_t, f(u)_t> = <dx_t, u_t>
    gen = torch.Generator(device="cuda").manual_seed(7)
    u = torch.randn(dp.x.shape, device="cuda", generator=gen).to(torch.bfloat16)
    y_u = torch.full_like(dp.y, float("nan"))
    plora.plora_linear_fwd(dp.desc, u, dp.W, dp.A, dp.B, y_u, None, dp.ws)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    res = fc.adjoint_per_row(dp.dy, y_u, dp.dx, u)
    say(f"  row-wise adjoint over {lay.T} rows: bad={res['n_bad']} worst={res['worst']:.3f} of the noise bound")
    assert res["n_bad"] == 0, res
    del u, y_u, dp
    torch.cuda.empty_cache()


@pytest.mark.parametrize("which", [0, 1], ids=["mlp_up", "mlp_down"])
def test_config3_full_size(which):
    check_full_size(wl.config(3)[which])


@pytest.mark.parametrize("which", range(7), ids=["q", "k", "v", "o", "gate", "up", "down"])
def test_config4_full_size(which):
    check_full_size(wl.config(4)[which])


@pytest.mark.parametrize("which", [0, 1], ids=["attn", "mlp_up"])
def test_config5_full_size(which):
    check_full_size(wl.config(5)[which])


def test_config5_mlp_up_full_size_weight_stored_out_in():
    """The largest linear with W stored [d_out][d_in]: the two GEMM forms in the other direction each, at full size."""
    from paper_2508_02932_amd import plora
    check_full_size(wl.config(5)[1], w_layout=plora.PLORA_W_OUT_IN)


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
    check_full_size(lin)
    # and with the roles of the hidden sizes swapped (wide contraction, narrow output)
    lin = wl.small("odd_many_tiles_T", "bf16", 4360, 1096,
                   lengths=[611, 1290, 3, 0, 977, 258, 1031, 307],
                   seg_adapter=[0, 1, 2, 3, -1, 4, 1, 5],
                   ranks=[128, 1, 24, 8, 72, 33], scales=[2.0, 0.5, 1.0, 4.0, 2.0, 0.25], seed=89)
    check_full_size(lin)
