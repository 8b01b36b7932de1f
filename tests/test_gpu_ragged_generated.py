"""Generated small ragged cases on the GPU (hypothesis, derandomised so that every run draws the
same cases): random segment counts and lengths (empty ones included), repeated and base-only
adapters, adapters without tokens, ranks anywhere in 1..128, hidden sizes that are multiples of 8
but of no tile.  Each case is compared element by element with the scalar-loop oracle.  No
shrinking and no second example after a failure: the run stops at the first failing case."""
import sys

import numpy as np
import pytest
from hypothesis import HealthCheck, Phase, given, settings, strategies as st

import oracle
from paper_2508_02932_amd import workloads as wl
from util import make_problem, scaled_err

pytestmark = pytest.mark.gpu
TOL = {"bf16": 2e-2, "f32": 1e-5}


@st.composite
def ragged_linear(draw):
    dtype = draw(st.sampled_from(["bf16", "bf16", "bf16", "f32"]))
    big = dtype == "bf16"
    D = 8 * draw(st.integers(1, 72 if big else 12))
    K = 8 * draw(st.integers(1, 72 if big else 12))
    n_ad = draw(st.integers(1, 5))
    ranks = [draw(st.sampled_from([1, 2, 7, 8, 16, 24, 33, 64, 100, 128])) for _ in range(n_ad)]
    scales = [draw(st.sampled_from([0.25, 0.5, 1.0, 2.0, 4.0])) for _ in range(n_ad)]
    n_seg = draw(st.integers(1, 7))
    max_len = 330 if big else 70
    lengths = [draw(st.one_of(st.just(0), st.integers(1, max_len))) for _ in range(n_seg)]
    seg_adapter = [draw(st.integers(-1, n_ad - 1)) for _ in range(n_seg)]
    seed = draw(st.integers(0, 999))
    return wl.small(f"gen_{dtype}_{seed}", dtype, D, K, lengths, seg_adapter, ranks, scales, seed=seed)


@settings(max_examples=24, deadline=None, derandomize=True, database=None, phases=[Phase.generate],
          report_multiple_bugs=False, suppress_health_check=list(HealthCheck))
@given(lin=ragged_linear(), save_h=st.booleans(), w_layout=st.sampled_from([0, 0, 1]))
def test_generated_ragged_cases(lin, save_h, w_layout):
    import torch
    import gpu_harness as gh
    lay = lin.layout
    print(f"[case] {lin.name} T={lay.T} D={lin.D} K={lin.K} ranks={lay.rank.tolist()} "
          f"segs={np.diff(lay.seg_off).tolist()} adapters={lay.seg_adapter.tolist()} save_h={save_h} "
          f"w_layout={w_layout}", flush=True)
    sys.stdout.flush()
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    y_o, h_o = oracle.loops.forward(p)
    dx_o, _, dA_o, dB_o = oracle.loops.backward(p, t.dy)
    dp = gh.upload(lin, t, w_layout)
    gh.forward(dp, save_h=save_h)
    gh.backward(dp, use_saved_h=save_h)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    tol = TOL[lin.dtype]
    errs = {}
    if lay.T:
        errs["y"] = scaled_err(gh.to_np(dp.y), y_o)
        errs["dx"] = scaled_err(gh.to_np(dp.dx), dx_o)
    if save_h and lay.sum_Lr() > 0:
        errs["h"] = scaled_err(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)[:lay.sum_Lr()]), h_o)
    for k in range(lay.n_adapters):
        errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o[k])
        errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o[k])
    for k, v in errs.items():
        assert np.isfinite(v) and v <= tol, (lin.name, k, v, tol)


@settings(max_examples=12, deadline=None, derandomize=True, database=None, phases=[Phase.generate],
          report_multiple_bugs=False, suppress_health_check=list(HealthCheck))
@given(lin=ragged_linear(), save_h=st.booleans())
def test_generated_ragged_cases_stand_alone_low_rank(lin, save_h):
    """The same generator through plora_lora_fwd / plora_lora_bwd: y and dx hold arbitrary values of the I/O type on
    entry and must come back as those values plus the oracle's low-rank term (the oracle run with W = 0)."""
    import torch
    import gpu_harness as gh
    lay = lin.layout
    print(f"[case] lora-only {lin.name} T={lay.T} D={lin.D} K={lin.K} ranks={lay.rank.tolist()} "
          f"segs={np.diff(lay.seg_off).tolist()} adapters={lay.seg_adapter.tolist()} save_h={save_h}", flush=True)
    sys.stdout.flush()
    t = lin.tensors()
    rng = np.random.default_rng(lay.T + 7)
    rnd = wl.round_to_bf16 if lin.dtype == "bf16" else (lambda a: a.astype(np.float32))
    y_in = rnd(rng.standard_normal((lay.T, lin.K)).astype(np.float32))
    dx_in = rnd(rng.standard_normal((lay.T, lin.D)).astype(np.float32))
    t.W = np.zeros_like(t.W)
    p0 = make_problem(oracle, lin, t)
    y_d, h_o = oracle.loops.forward(p0)
    dx_d, _, dA_o, dB_o = oracle.loops.backward(p0, t.dy)
    dp = gh.upload(lin, t, lora_only=True)
    dp.y.copy_(gh.to_dev(y_in, lin.dtype))
    dp.dx.copy_(gh.to_dev(dx_in, lin.dtype))
    gh.lora_forward(dp, save_h=save_h)
    gh.lora_backward(dp, use_saved_h=save_h)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    tol = TOL[lin.dtype]
    errs = {}
    if lay.T:
        errs["y"] = scaled_err(gh.to_np(dp.y), y_in.astype(np.float64) + y_d)
        errs["dx"] = scaled_err(gh.to_np(dp.dx), dx_in.astype(np.float64) + dx_d)
    if save_h and lay.sum_Lr() > 0:
        errs["h"] = scaled_err(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)[:lay.sum_Lr()]), h_o)
    for k in range(lay.n_adapters):
        errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o[k])
        errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o[k])
    for k, v in errs.items():
        assert np.isfinite(v) and v <= tol, (lin.name, k, v, tol)


@st.composite
def ragged_group(draw):
    """2 to 4 projections on one x and one packing; widths, ranks, scales, weight layouts and the per-projection options
    (saved activation, weight gradients, dx) drawn independently."""
    n_proj = draw(st.integers(2, 4))
    D = 8 * draw(st.integers(1, 72))
    n_ad = draw(st.integers(1, 4))
    n_seg = draw(st.integers(1, 6))
    lengths = [draw(st.sampled_from([130, 0, 1, 64, 127, 129, 300, 513])) for _ in range(n_seg)]
    seg_adapter = [draw(st.sampled_from([0, -1] + list(range(n_ad)))) for _ in range(n_seg)]
    seed = draw(st.integers(0, 999))
    lins, opts = [], []
    for p in range(n_proj):
        K = 8 * draw(st.integers(1, 40))
        ranks = [draw(st.sampled_from([16, 1, 7, 8, 16, 24, 33, 48, 64, 100])) for _ in range(n_ad)]
        scales = [draw(st.sampled_from([0.25, 0.5, 1.0, 2.0])) for _ in range(n_ad)]
        lins.append(wl.small(f"ggen_{seed}_p{p}", "bf16", D, K, lengths, seg_adapter, ranks, scales, seed=7 * seed + p))
        opts.append((draw(st.sampled_from([0, 1])), draw(st.booleans()), draw(st.sampled_from([True, True, True, False])),
                     draw(st.sampled_from([True, True, False]))))
    if draw(st.sampled_from([False, False, True])):      # one time in three: the summed input gradient instead of one dx each
        opts = [o[:3] + ("sum",) for o in opts]
    return lins, opts


@settings(max_examples=20, deadline=None, derandomize=True, database=None, phases=[Phase.generate],
          report_multiple_bugs=False, suppress_health_check=list(HealthCheck))
@given(case=ragged_group())
def test_generated_ragged_groups(case):
    """The same kind of generated packing through plora_group_fwd / plora_group_bwd: every projection against the oracle
    for that projection alone; outputs that were not asked for stay untouched."""
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    lins, opts = case
    lay = lins[0].layout
    print(f"[case] group D={lins[0].D} K={[l.K for l in lins]} T={lay.T} ranks={[l.layout.rank.tolist() for l in lins]} "
          f"segs={np.diff(lay.seg_off).tolist()} adapters={lay.seg_adapter.tolist()} (w_layout, save_h, want_w, want_dx)={opts}",
          flush=True)
    sys.stdout.flush()
    tens = [l.tensors() for l in lins]
    for t in tens[1:]:
        t.x = tens[0].x
    dps = [gh.upload(l, t, o[0]) for l, t, o in zip(lins, tens, opts)]
    group = plora.Group([dp.desc for dp in dps])
    guards: list = []
    ws = gh.guarded((plora.plora_group_workspace_bytes(group),), torch.uint8, None, guards, "group workspace")
    pick = lambda items, flags: [it if f else None for it, f in zip(items, flags)] if any(flags) else None
    save_h, want_w, want_dx = ([o[i] for o in opts] for i in (1, 2, 3))
    use_sum = want_dx[0] == "sum"
    dx_sum = gh.guarded(tuple(dps[0].dx.shape), torch.bfloat16, float("nan"), guards, "dx_sum") if use_sum else None
    if use_sum:
        want_dx = [False] * len(opts)
    h = pick([dp.h for dp in dps], save_h)
    plora.plora_group_fwd(group, dps[0].x, [dp.W for dp in dps], [dp.A for dp in dps], [dp.B for dp in dps],
                          [dp.y for dp in dps], h, ws)
    plora.plora_group_bwd(group, dps[0].x, [dp.W for dp in dps], [dp.A for dp in dps], [dp.B for dp in dps],
                          [dp.dy for dp in dps], h, pick([dp.dx for dp in dps], want_dx), pick([dp.dA for dp in dps], want_w),
                          pick([dp.dB for dp in dps], want_w), ws, dx_sum=dx_sum)
    torch.cuda.synchronize()
    for name, base, nbytes in guards:
        assert bool((base[:gh.GUARD_BYTES] == gh.GUARD_BYTE).all()) and bool((base[gh.GUARD_BYTES + nbytes:] == gh.GUARD_BYTE).all()), name
    dx_total = np.zeros((lay.T, lins[0].D), dtype=np.float64)
    for p, (lin, t, dp) in enumerate(zip(lins, tens, dps)):
        gh.check_guards(dp)
        prob = make_problem(oracle, lin, t)
        y_o, h_o = oracle.loops.forward(prob)
        dx_o, _, dA_o, dB_o = oracle.loops.backward(prob, t.dy)
        dx_total += dx_o
        errs = {}
        if lay.T:
            errs["y"] = scaled_err(gh.to_np(dp.y), y_o)
            if want_dx[p]:
                errs["dx"] = scaled_err(gh.to_np(dp.dx), dx_o)
            else:
                assert bool(dp.dx.float().isnan().all()), (p, "dx written")
        if save_h[p] and lay.sum_Lr() > 0:
            errs["h"] = scaled_err(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)[:lin.layout.sum_Lr()]), h_o)
        for k in range(lay.n_adapters):
            if want_w[p]:
                errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o[k])
                errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o[k])
            else:
                assert bool(dp.dA[k].isnan().all()) and bool(dp.dB[k].isnan().all()), (p, k, "gradients written")
        for k, v in errs.items():
            assert np.isfinite(v) and v <= TOL["bf16"], (lin.name, p, k, v)
    if use_sum and lay.T:
        v = scaled_err(gh.to_np(dx_sum), dx_total)
        assert np.isfinite(v) and v <= TOL["bf16"], ("dx_sum", v)
