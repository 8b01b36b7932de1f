"""GPU parity of the stand-alone low-rank calls (plora_lora_fwd / plora_lora_bwd): the caller's buffers hold the base
products x W and dy W^T, the library adds scale_k (x A_k) B_k and g A_k^T in place (section 2.4; appendix C.2, case 4)
and writes dA_k, dB_k (cases 3 and 1).  Expected values: the given base (as the library reads it, already rounded to
the I/O type) plus the oracle's low-rank term, which is the oracle run with W = 0; weight gradients and the saved
activation do not depend on W at all.  Rows of segments without an adapter must come back bit for bit."""
import numpy as np
import pytest

import oracle
from paper_2508_02932_amd import workloads as wl
from util import make_problem, scaled_err
from test_gpu_parity import TOL, say

pytestmark = pytest.mark.gpu


def run_lora_only(lin, t=None, impl=None, save_h=True, want_dx=True, exact=False):
    import torch
    import gpu_harness as gh
    t = t or lin.tensors()
    impl = impl or oracle.loops
    tol = 0.0 if exact else TOL[lin.dtype]
    lay = lin.layout
    say(f"[case] lora-only {lin.name} dtype={lin.dtype} T={lay.T} D={lin.D} K={lin.K} ranks={lay.rank.tolist()} "
        f"segs={np.diff(lay.seg_off).tolist()} adapters={lay.seg_adapter.tolist()} save_h={save_h} dx={want_dx}")
    # base products as a caller's own GEMM would leave them: any values of the I/O type will do; take the true ones
    rnd = wl.round_to_bf16 if lin.dtype == "bf16" else (lambda a: a.astype(np.float32))
    y_in = rnd((t.x.astype(np.float64) @ t.W.astype(np.float64)).astype(np.float32))
    dx_in = rnd((t.dy.astype(np.float64) @ t.W.astype(np.float64).T).astype(np.float32))
    p = make_problem(oracle, lin, t)
    t0 = lin.tensors()
    t0.x, t0.A, t0.B, t0.dy = t.x, t.A, t.B, t.dy
    t0.W = np.zeros_like(t.W)
    p0 = make_problem(oracle, lin, t0)
    y_delta, h_o = impl.forward(p0)
    dx_delta, _, dA_o, dB_o = impl.backward(p0, t.dy)
    y_o = y_in.astype(np.float64) + y_delta
    dx_o = dx_in.astype(np.float64) + dx_delta
    if exact:       # the sums are exact in fp32; what is left is the one rounding to the I/O type
        y_o = rnd(y_o.astype(np.float32)).astype(np.float64)
        dx_o = rnd(dx_o.astype(np.float32)).astype(np.float64)

    dp = gh.upload(lin, t, lora_only=True)
    dp.y.copy_(gh.to_dev(y_in, lin.dtype))
    dp.dx.copy_(gh.to_dev(dx_in, lin.dtype))
    say("  forward")
    gh.lora_forward(dp, save_h=save_h)
    torch.cuda.synchronize()
    say("  backward")
    gh.lora_backward(dp, use_saved_h=save_h, want_dx=want_dx)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    y, dx = gh.to_np(dp.y), gh.to_np(dp.dx)
    errs = {"y": scaled_err(y, y_o)}
    if want_dx:
        errs["dx"] = scaled_err(dx, dx_o)
    else:
        assert np.array_equal(dx, dx_in)                          # untouched
    if save_h and lay.sum_Lr() > 0:
        errs["h"] = scaled_err(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)[:lay.sum_Lr()]), h_o)
    for k in range(lay.n_adapters):
        errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o[k])
        errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o[k])
    say("  errors " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    for k, v in errs.items():
        assert np.isfinite(v) and v <= tol, (lin.name, k, v, tol)
    # rows without an adapter are not touched
    for s in range(lay.n_seg):
        if int(lay.seg_adapter[s]) < 0:
            lo, hi = int(lay.seg_off[s]), int(lay.seg_off[s + 1])
            assert np.array_equal(y[lo:hi], y_in[lo:hi]) and np.array_equal(dx[lo:hi], dx_in[lo:hi])
    return dp


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_lora_only_ragged_small(dtype):
    lin = wl.small(f"lo_ragged_{dtype}", dtype, 328, 264, lengths=[130, 0, 257, 64, 249, 1],
                   seg_adapter=[1, 0, 2, -1, 1, 0], ranks=[8, 24, 72], scales=[2.0, 0.5, 1.25], seed=341)
    run_lora_only(lin)


def test_lora_only_several_tiles():
    """Several column tiles of 128 with a ragged last one in both directions, rank 1, odd rank, maximum rank, a token
    block with a single row."""
    lin = wl.small("lo_tiles", "bf16", 576, 520, lengths=[200, 90, 310, 7, 129],
                   seg_adapter=[0, 1, 2, 3, 0], ranks=[128, 1, 33, 64], scales=[2.0, 4.0, 0.25, 1.0], seed=347)
    run_lora_only(lin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_lora_only_without_saved_h_and_without_dx(dtype):
    lin = wl.small(f"lo_recompute_{dtype}", dtype, 256, 192, lengths=[100, 300], seg_adapter=[0, 1],
                   ranks=[16, 40], scales=[2.0, 2.0], seed=343)
    run_lora_only(lin, save_h=False, want_dx=False)


def test_lora_only_exact_integers():
    """Small-integer inputs and power-of-two scales: every product and sum is exact in bf16 / fp32, so the update
    must equal the oracle with zero error (indexing, masks and the single rounding, free of tolerance)."""
    lin = wl.small("lo_exact", "bf16", 136, 264, lengths=[70, 3, 130, 64], seg_adapter=[0, -1, 1, 0], ranks=[3, 16],
                   scales=[2.0, 0.5], seed=349)
    rng = np.random.default_rng(7)
    t = lin.tensors()
    t.x = rng.integers(-1, 2, size=t.x.shape).astype(np.float32)
    t.dy = rng.integers(-1, 2, size=t.dy.shape).astype(np.float32)
    t.W = rng.integers(-1, 2, size=t.W.shape).astype(np.float32)
    t.A = [rng.integers(-1, 2, size=a.shape).astype(np.float32) for a in t.A]
    t.B = [rng.integers(-1, 2, size=b.shape).astype(np.float32) for b in t.B]
    run_lora_only(lin, t, exact=True)


def test_lora_only_edge_cases():
    import torch
    import gpu_harness as gh
    lin = wl.small("lo_edge", "bf16", 64, 72, lengths=[1, 0, 5], seg_adapter=[0, 1, -1], ranks=[4, 16],
                   scales=[1.0, 3.0], seed=361)
    run_lora_only(lin)
    lin = wl.small("lo_base_only", "bf16", 64, 64, lengths=[70], seg_adapter=[-1], ranks=[8], scales=[1.0], seed=367)
    run_lora_only(lin)
    lin = wl.small("lo_empty", "bf16", 64, 64, lengths=[0], seg_adapter=[0], ranks=[8], scales=[1.0], seed=371)
    dp = gh.upload(lin, lin.tensors(), lora_only=True)
    gh.lora_forward(dp)
    gh.lora_backward(dp)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    assert not gh.to_np(dp.dA[0]).any() and not gh.to_np(dp.dB[0]).any()


def test_lora_only_config2_full():
    run_lora_only(wl.config(2)[0], impl=oracle.matmul)


def test_lora_only_errors():
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    lin = wl.small("lo_err", "bf16", 64, 64, lengths=[8], seg_adapter=[0], ranks=[8], scales=[1.0], seed=1)
    dp = gh.upload(lin, lin.tensors(), lora_only=True)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(plora.PloraError) as e:
        plora.plora_lora_fwd(dp.desc, dp.x, dp.A, dp.B, dp.y, None, small)
    assert e.value.code == 7                                      # PLORA_ERR_WORKSPACE
    with pytest.raises(plora.PloraError) as e:
        plora.plora_lora_fwd(dp.desc, dp.x, dp.A, dp.B, None, None, dp.ws)
    assert e.value.code == 1                                      # PLORA_ERR_NULL


def test_lora_only_config5_mlp_up_full_size():
    """The largest linear through the stand-alone calls, in the launch configuration bench.py times: h, dA_k, dB_k of
    every adapter in full; y and dx on two whole 256-row tiles, the rows around every segment boundary and random rows
    against the oracle (run with W = 0 on those rows, added to what the buffers held); every other row must differ
    from its input by a finite amount, and rows without an adapter not at all (there are none here, but the base
    values of all rows are kept for the comparison)."""
    import time
    import torch
    import gpu_harness as gh
    import fullsize_checks as fc
    lin = wl.config(5)[1]
    lay = lin.layout
    t = lin.tensors()
    say(f"[case] lora-only {lin.name} T={lay.T} D={lin.D} K={lin.K}")
    dp = gh.upload(lin, t, lora_only=True)
    gen = torch.Generator(device="cuda").manual_seed(11)
    y_in = torch.randn(dp.y.shape, device="cuda", generator=gen).to(torch.bfloat16)
    dx_in = torch.randn(dp.dx.shape, device="cuda", generator=gen).to(torch.bfloat16)
    dp.y.copy_(y_in)
    dp.dx.copy_(dx_in)
    gh.lora_forward(dp)
    gh.lora_backward(dp)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    p = make_problem(oracle, lin, t)
    errs = {"h": fc.compare(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)), oracle.matmul.low_rank_activation(p))}
    dA_o, dB_o = oracle.matmul.low_rank_gradients(p, t.dy)
    for k in range(lay.n_adapters):
        errs[f"dA{k}"] = fc.compare(gh.to_np(dp.dA[k]), dA_o[k])
        errs[f"dB{k}"] = fc.compare(gh.to_np(dp.dB[k]), dB_o[k])
    rows = fc.plan_rows(lay.seg_off, 2, 64, np.random.default_rng(3))
    t0 = time.time()
    t.W = np.zeros_like(t.W)
    sub = make_problem(oracle, lin, t).take_rows(rows)
    y_d, _ = oracle.matmul.forward(sub)
    dx_d, _, _, _ = oracle.matmul.backward(sub, t.dy[rows])
    say(f"  oracle: low-rank terms of {len(rows)} rows in {time.time() - t0:.1f} s")
    idx = torch.from_numpy(rows).cuda()
    errs["y"] = fc.compare(gh.to_np(dp.y[idx]), gh.to_np(y_in[idx]).astype(np.float64) + y_d)
    errs["dx"] = fc.compare(gh.to_np(dp.dx[idx]), gh.to_np(dx_in[idx]).astype(np.float64) + dx_d)
    say("  errors " + " ".join(f"{k}={v:.2e}" for k, v in errs.items() if k in ("h", "y", "dx")) + f" max {max(errs.values()):.2e}")
    assert all(np.isfinite(v) and v <= TOL["bf16"] for v in errs.values()), errs
    # every row was updated by something finite and of the size of a low-rank term, none was skipped or overwritten
    dy_rows = (dp.y.float() - y_in.float()).abs().amax(dim=1)
    ddx_rows = (dp.dx.float() - dx_in.float()).abs().amax(dim=1)
    assert bool(torch.isfinite(dy_rows).all()) and bool(torch.isfinite(ddx_rows).all())
    assert float(dy_rows.min()) > 0 and float(ddx_rows.min()) > 0
    assert float(dy_rows.max()) < 64 and float(ddx_rows.max()) < 64
