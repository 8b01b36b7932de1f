"""GPU parity: the HIP library against the fp64 CPU oracle, element by element, on the same seeded
inputs.  Sizes here are ones the oracle finishes in seconds, yet they span several tiles of every
kernel and have ragged tails.  Tolerances (scaled error, see util.scaled_err): 2e-2 for bf16 I/O
with fp32 accumulation, 1e-5 for fp32 I/O; segment indexing is implicit in every comparison (a
wrong row or adapter is an O(1) error)."""
import sys

import numpy as np
import pytest

import oracle
from paper_2508_02932_amd import workloads as wl
from util import make_problem, scaled_err

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "f32": 1e-5}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_and_compare(lin, t=None, impl=None, save_h=True, check_h=True, w_layout=0):
    import torch
    import gpu_harness as gh
    t = t or lin.tensors()
    impl = impl or oracle.loops
    tol = TOL[lin.dtype]
    say(f"[case] {lin.name} dtype={lin.dtype} T={lin.layout.T} D={lin.D} K={lin.K} "
        f"ranks={lin.layout.rank.tolist()} segs={np.diff(lin.layout.seg_off).tolist()} "
        f"adapters={lin.layout.seg_adapter.tolist()} save_h={save_h} w_layout={w_layout}")
    p = make_problem(oracle, lin, t)
    y_o, h_o = impl.forward(p)
    dx_o, g_o, dA_o, dB_o = impl.backward(p, t.dy)

    dp = gh.upload(lin, t, w_layout)
    say("  forward")
    gh.forward(dp, save_h=save_h)
    torch.cuda.synchronize()
    say("  backward")
    gh.backward(dp, use_saved_h=save_h)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    y = gh.to_np(dp.y)
    dx = gh.to_np(dp.dx)
    errs = {"y": scaled_err(y, y_o), "dx": scaled_err(dx, dx_o)}
    if save_h and check_h and lin.layout.sum_Lr() > 0:
        h = gh.ragged_h_to_rows(lin, gh.to_np(dp.h)[:lin.layout.sum_Lr()])
        errs["h"] = scaled_err(h, h_o)
    for k in range(lin.layout.n_adapters):
        errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o[k])
        errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o[k])
    say("  errors " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    for k, v in errs.items():
        assert np.isfinite(v) and v <= tol, (lin.name, k, v, tol)
    return dp, errs


def test_config1_fp32_full():
    run_and_compare(wl.config(1)[0])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_small(dtype):
    """Repeated adapter, base-only segment, empty segment, segment lengths that are no multiple of
    any tile, D and K that are multiples of 8 only."""
    lin = wl.small(f"ragged_{dtype}", dtype, 328, 264, lengths=[130, 0, 257, 64, 249, 1],
                   seg_adapter=[1, 0, 2, -1, 1, 0], ranks=[8, 24, 72], scales=[2.0, 0.5, 1.25], seed=41)
    run_and_compare(lin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recompute_h_path(dtype):
    """Backward without the saved activation recomputes x A_k."""
    lin = wl.small(f"recompute_{dtype}", dtype, 256, 192, lengths=[100, 300], seg_adapter=[0, 1],
                   ranks=[16, 40], scales=[2.0, 2.0], seed=43)
    run_and_compare(lin, save_h=False)


def test_bf16_several_tiles():
    """More than one 256x256 GEMM tile in both directions, tiles that straddle three segments,
    rank 1 and the maximum rank 128, odd rank."""
    lin = wl.small("tiles_bf16", "bf16", 576, 520, lengths=[200, 90, 310, 7, 180],
                   seg_adapter=[0, 1, 2, 3, 0], ranks=[128, 1, 33, 64], scales=[2.0, 4.0, 0.25, 1.0], seed=47)
    run_and_compare(lin)


def test_bf16_pure_lora_delta():
    """W = 0 isolates the low-rank path, so its error is measured against its own magnitude."""
    lin = wl.small("w0_bf16", "bf16", 512, 512, lengths=[300, 212], seg_adapter=[1, 0], ranks=[16, 64],
                   scales=[2.0, 2.0], seed=53)
    t = lin.tensors()
    t.W = np.zeros_like(t.W)
    run_and_compare(lin, t)


def test_bf16_zero_B():
    lin = wl.small("b0_bf16", "bf16", 256, 256, lengths=[128, 128], seg_adapter=[0, 1], ranks=[8, 32],
                   scales=[2.0, 2.0], seed=59)
    t = lin.tensors()
    t.B = [np.zeros_like(b) for b in t.B]
    dp, _ = run_and_compare(lin, t)
    import gpu_harness as gh
    for k in range(2):
        assert not gh.to_np(dp.dA[k]).any()      # exactly zero, as in the oracle


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_edge_cases(dtype):
    import torch
    import gpu_harness as gh
    # adapter without tokens, all-base batch, single token
    lin = wl.small(f"edge_{dtype}", dtype, 64, 72, lengths=[1, 0, 5], seg_adapter=[0, 1, -1], ranks=[4, 16],
                   scales=[1.0, 3.0], seed=61)
    dp, _ = run_and_compare(lin)
    assert not gh.to_np(dp.dA[1]).any() and not gh.to_np(dp.dB[1]).any()
    lin = wl.small(f"base_only_{dtype}", dtype, 64, 64, lengths=[70], seg_adapter=[-1], ranks=[8], scales=[1.0], seed=67)
    run_and_compare(lin)
    # empty batch: forward is a no-op, backward writes zero weight gradients
    lin = wl.small(f"empty_{dtype}", dtype, 64, 64, lengths=[0], seg_adapter=[0], ranks=[8], scales=[1.0], seed=71)
    say(f"[case] {lin.name}")
    t = lin.tensors()
    dp = gh.upload(lin, t)
    gh.forward(dp)
    gh.backward(dp)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    assert not gh.to_np(dp.dA[0]).any() and not gh.to_np(dp.dB[0]).any()


def test_skip_outputs():
    """dx = NULL and dA = dB = NULL are honoured (the skipped outputs keep their NaN fill)."""
    import torch
    import gpu_harness as gh
    lin = wl.small("skip_bf16", "bf16", 128, 128, lengths=[96, 64], seg_adapter=[0, 1], ranks=[8, 16],
                   scales=[2.0, 2.0], seed=73)
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    dx_o, _, dA_o, dB_o = oracle.loops.backward(p, t.dy)
    dp = gh.upload(lin, t)
    say("[case] skip dx")
    gh.forward(dp)
    gh.backward(dp, want_dx=False)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    assert np.isnan(gh.to_np(dp.dx)).all()
    assert scaled_err(gh.to_np(dp.dA[1]), dA_o[1]) < 2e-2
    dp = gh.upload(lin, t)
    say("[case] skip dA/dB")
    gh.forward(dp)
    gh.backward(dp, want_w=False)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    assert np.isnan(gh.to_np(dp.dA[0])).all() and np.isnan(gh.to_np(dp.dB[1])).all()
    assert scaled_err(gh.to_np(dp.dx), dx_o) < 2e-2


def test_bf16_exact_integers():
    """Small-integer inputs: every product and partial sum is exact in bf16 x bf16 -> fp32, and the
    bf16 intermediates (h, g) are integers below 256, so the GPU must match the oracle with zero
    error after the final rounding."""
    import torch
    import gpu_harness as gh
    rng = np.random.default_rng(5)
    D = K = 256
    lens = [70, 130, 56]
    ranks = [4, 8]

    def sparse(shape):
        return (rng.integers(-1, 2, size=shape) * (rng.random(shape) < 0.125)).astype(np.float32)

    lin = wl.small("exact_bf16", "bf16", D, K, lengths=lens, seg_adapter=[0, 1, 0], ranks=ranks, scales=[1.0, 2.0])
    T = sum(lens)
    t = wl.Tensors(sparse((T, D)), sparse((D, K)), [sparse((D, r)) for r in ranks],
                   [sparse((r, K)) for r in ranks], sparse((T, K)))
    p = make_problem(oracle, lin, t)
    y_o, _ = oracle.loops.forward(p)
    dx_o, _, dA_o, dB_o = oracle.loops.backward(p, t.dy)
    say("[case] exact integers")
    dp = gh.upload(lin, t)
    gh.forward(dp)
    gh.backward(dp)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    assert np.array_equal(gh.to_np(dp.y), wl.round_to_bf16(y_o.astype(np.float32)))
    assert np.array_equal(gh.to_np(dp.dx), wl.round_to_bf16(dx_o.astype(np.float32)))
    for k in range(2):
        assert np.array_equal(gh.to_np(dp.dA[k]), dA_o[k].astype(np.float32))
        assert np.array_equal(gh.to_np(dp.dB[k]), dB_o[k].astype(np.float32))


def test_run_twice_bitwise_identical():
    """No atomics and a fixed summation order: two runs give the same bits."""
    import torch
    import gpu_harness as gh
    lin = wl.small("twice_bf16", "bf16", 512, 384, lengths=[333, 190, 77], seg_adapter=[0, 1, 0], ranks=[24, 64],
                   scales=[2.0, 2.0], seed=79)
    t = lin.tensors()
    outs = []
    for rep in range(2):
        say(f"[case] run twice, run {rep}")
        dp = gh.upload(lin, t)
        gh.forward(dp)
        gh.backward(dp)
        torch.cuda.synchronize()
        outs.append([gh.to_np(dp.y), gh.to_np(dp.dx)] + [gh.to_np(a) for a in dp.dA] + [gh.to_np(b) for b in dp.dB])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_side_stream_and_workspace_reuse():
    """The calls enqueue on the stream they are given (here a second stream of default priority, with the
    inputs produced on it) and leave nothing behind in the workspace that a later call with another
    description depends on: two different problems alternate on one workspace and one stream and each
    keeps giving its own bits."""
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    lin_a = wl.small("stream_a", "bf16", 320, 264, lengths=[150, 0, 221], seg_adapter=[1, 0, 0], ranks=[40, 8],
                     scales=[1.0, 2.0], seed=97)
    lin_b = wl.small("stream_b", "bf16", 264, 320, lengths=[97, 130], seg_adapter=[0, -1], ranks=[128],
                     scales=[0.5], seed=101)
    ref = {}
    for lin in (lin_a, lin_b):                                   # reference bits on the default stream
        dp, _ = run_and_compare(lin)
        ref[lin.name] = [gh.to_np(dp.y), gh.to_np(dp.dx)] + [gh.to_np(a) for a in dp.dA] + [gh.to_np(b) for b in dp.dB]
    side = torch.cuda.Stream()
    dps = {lin.name: gh.upload(lin, lin.tensors()) for lin in (lin_a, lin_b)}
    ws = torch.empty(max(d.ws.numel() for d in dps.values()), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for rep in range(3):
            for name, dp in dps.items():
                say(f"[case] side stream, rep {rep}, {name}")
                plora.plora_linear_fwd(dp.desc, dp.x, dp.W, dp.A, dp.B, dp.y, dp.h, ws, stream=side)
                plora.plora_linear_bwd(dp.desc, dp.x, dp.W, dp.A, dp.B, dp.dy, dp.h, dp.dx, dp.dA, dp.dB, ws, stream=side)
    side.synchronize()
    for name, dp in dps.items():
        gh.check_guards(dp)
        got = [gh.to_np(dp.y), gh.to_np(dp.dx)] + [gh.to_np(a) for a in dp.dA] + [gh.to_np(b) for b in dp.dB]
        for a, b in zip(got, ref[name]):
            assert np.array_equal(a, b), name


def _device_tables_equal_export(lin, w_layout=0):
    """The tables the preparation kernel derived in the workspace are, byte for byte, the ones the host
    exports (and the brute-force tests check), adapter pointers aside."""
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    t = lin.tensors()
    dp = gh.upload(lin, t, w_layout)
    gh.forward(dp)
    gh.backward(dp)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    info, tabs, image = plora.plora_debug_metadata(dp.desc)
    dev = dp.ws[info.ws_meta:info.ws_meta + info.table_bytes].cpu().numpy()
    got = plora.parse_tables(info, dev)
    for k in range(lin.layout.n_adapters):      # the device copy carries this call's pointers
        assert int(got["ad"][k]["A"]) == dp.A[k].data_ptr() and int(got["ad"][k]["dB"]) == dp.dB[k].data_ptr()
    at_base = dp.ws.data_ptr() + info.ws_at
    assert int(got["hdr"]["at_base"]) == at_base
    for k in range(lin.layout.n_adapters):      # the [r][N] low-rank operand: B_k, or the packed A_k^T
        want = at_base + 2 * int(got["ad"][k]["at_off"]) if w_layout else dp.B[k].data_ptr()
        assert int(got["ad"][k]["ext_b"]) == want
    for rec in got["tile"]:                     # a tile's first record names the operand of its first segment's adapter
        if int(rec["n_own"]) > 0:
            a = int(got["seg"][int(rec["first_seg"])]["adapter"])
            assert int(rec["s"][0]["B"]) == int(got["ad"][a]["ext_b"])
    for name in ("A", "B", "dA", "dB", "ext_b"):
        got["ad"][name] = 0
        tabs["ad"][name] = 0
    got["tile"]["s"]["B"] = 0
    tabs["tile"]["s"]["B"] = 0
    got["hdr"]["at_base"] = 0
    assert got["hdr"] == tabs["hdr"]
    for name in ("seg", "ad", "tile", "blk_seg", "seg_list", "tile_order"):
        assert np.array_equal(got[name], tabs[name]), name
    return dp


def test_device_tables_equal_host_export():
    lin = wl.small("tables_dev", "bf16", 328, 264, lengths=[130, 0, 257, 64, 249, 1, 700, 30, 12],
                   seg_adapter=[1, 0, 2, -1, 1, 0, 3, 2, 0], ranks=[8, 24, 72, 128], scales=[2.0, 0.5, 1.25, 1.0], seed=151)
    _device_tables_equal_export(lin)


def test_many_adapters_chunked_description():
    """More adapters than one kernel argument carries (the description is uploaded in chunks first):
    same tables, same results."""
    n_ad = 100
    rng = np.random.default_rng(9)
    lengths = rng.integers(0, 40, size=120).tolist()
    seg_adapter = rng.integers(-1, n_ad, size=120).tolist()
    ranks = rng.integers(1, 33, size=n_ad).tolist()
    lin = wl.small("many_adapters", "bf16", 136, 264, lengths=lengths, seg_adapter=seg_adapter, ranks=ranks,
                   scales=[1.0] * n_ad, seed=157)
    from paper_2508_02932_amd import plora
    import gpu_harness as gh
    info, _, _ = plora.plora_debug_metadata(gh.desc_of(lin))
    assert info.desc_words > 896
    _device_tables_equal_export(lin)
    run_and_compare(lin)


def test_most_adapters_and_segments():
    """The largest description the interface takes: 256 adapters, 1024 segments (many of them empty or a few rows
    long), so that the description travels in several chunks and the segment table no longer fits the preparation
    kernel's LDS copy."""
    from paper_2508_02932_amd import plora
    import gpu_harness as gh
    n_ad, n_seg = 256, 1024
    rng = np.random.default_rng(19)
    lengths = rng.integers(0, 12, size=n_seg)
    lengths[rng.integers(0, n_seg, size=40)] = rng.integers(100, 400, size=40)      # some long enough for several blocks
    seg_adapter = rng.integers(-1, n_ad, size=n_seg)
    ranks = rng.integers(1, 129, size=n_ad)
    lin = wl.small("most_adapters", "bf16", 72, 136, lengths=lengths.tolist(), seg_adapter=seg_adapter.tolist(),
                   ranks=ranks.tolist(), scales=[0.5] * n_ad, seed=163)
    info, _, _ = plora.plora_debug_metadata(gh.desc_of(lin))
    assert info.desc_words > 3 * 896
    _device_tables_equal_export(lin)
    run_and_compare(lin, impl=oracle.matmul)


def test_tall_batch():
    """Several hundred thousand token rows against a narrow layer: thousands of GEMM row tiles and token blocks (the
    tile order, the block table and every 64-bit row offset at a size the configurations never reach)."""
    rng = np.random.default_rng(23)
    lengths = [150_001, 0, 99_999, 250_000, 37, 100_003]
    lin = wl.small("tall", "bf16", 16, 24, lengths=lengths, seg_adapter=[0, 1, 2, -1, 1, 0], ranks=[8, 128, 40],
                   scales=[2.0, 1.0, 0.5], seed=167)
    run_and_compare(lin, impl=oracle.matmul)
