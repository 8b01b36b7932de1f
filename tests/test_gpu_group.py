"""Grouped calls (several projections on one x: plora_group_fwd / plora_group_bwd) on the GPU.

A projection of a group is an ordinary layer of its own, so the expected values are the oracle's for every projection
alone (appendix C.2: concatenating adapters changes the traffic, not the results).  The cases cover one fused pass
over all projections, groups that are cut into several passes because the ranks do not fit one, groups that cannot be
fused at all, projections that differ in width, rank, scale and weight layout, and per-projection options (no saved
activation, no weight gradients, no dx)."""
import sys

import numpy as np
import pytest

import oracle
from paper_2508_02932_amd import workloads as wl
from util import make_problem, scaled_err

pytestmark = pytest.mark.gpu
TOL = {"bf16": 2e-2, "f32": 1e-5}


def make_group(dtype, D, Ks, lengths, seg_adapter, ranks_per_proj, scales_per_proj, seed):
    """Projections with one x and one packing; each has its own width, ranks, scales, W, A, B and dy."""
    lins, tens = [], []
    for p, K in enumerate(Ks):
        lin = wl.small(f"grp{seed}_p{p}", dtype, D, K, lengths, seg_adapter, ranks_per_proj[p], scales_per_proj[p],
                       seed=100 * seed + p)
        t = lin.tensors()
        if p:
            t.x = tens[0].x
        lins.append(lin)
        tens.append(t)
    return lins, tens


CASES = {
    # one fused pass over three projections (sums of padded ranks: 64, 64, 112)
    "qkv_one_pass": dict(dtype="bf16", D=320, Ks=(256, 64, 72), lengths=(130, 0, 257, 64, 300), seg_adapter=(0, 1, 2, -1, 1),
                         ranks=((8, 16, 33), (16, 16, 7), (24, 32, 40)), scales=((2.0, 1.0, 0.5), (1.0, 0.25, 2.0), (0.5, 0.5, 4.0))),
    # rank 64 everywhere: the first two projections fill a pass, the third runs alone
    "cut_in_two": dict(dtype="bf16", D=256, Ks=(128, 128, 192), lengths=(200, 129), seg_adapter=(1, 0),
                       ranks=((64, 64), (64, 50), (64, 64)), scales=((1.0, 1.0), (2.0, 0.5), (1.0, 0.25))),
    # rank 128: nothing can be fused
    "no_fusion": dict(dtype="bf16", D=128, Ks=(64, 64), lengths=(150,), seg_adapter=(0,),
                      ranks=((128,), (100,)), scales=((1.0,), (1.0,))),
    # four projections, an adapter without tokens, a repeated adapter, base-only rows
    "four": dict(dtype="bf16", D=520, Ks=(64, 128, 8, 264), lengths=(70, 5, 640, 33, 128), seg_adapter=(2, -1, 0, 2, 0),
                 ranks=((1, 16, 16), (16, 128, 17), (32, 8, 30), (9, 64, 2)), scales=((1.0,) * 3,) * 4),
    # two wide projections that need contraction splits in the fused passes
    "gate_up": dict(dtype="bf16", D=2048, Ks=(512, 512), lengths=(256, 384, 100), seg_adapter=(0, 1, 0),
                    ranks=((16, 64), (48, 64)), scales=((2.0, 2.0), (2.0, 2.0))),
    # long segments: the fused dA pass splits its token walk and sums partial tiles
    "long": dict(dtype="bf16", D=512, Ks=(128, 64), lengths=(4096, 4000), seg_adapter=(0, 1),
                 ranks=((64, 32), (64, 96)), scales=((1.0, 2.0), (0.5, 1.0))),
    # more adapters than one kernel argument carries: the description takes the chunked upload path in every projection
    "many_adapters": dict(dtype="bf16", D=136, Ks=(72, 200), lengths=tuple(3 + (7 * i) % 41 for i in range(140)),
                          seg_adapter=tuple((11 * i) % 100 for i in range(140)),
                          ranks=(tuple(1 + (5 * k) % 40 for k in range(100)), tuple(8 + (3 * k) % 50 for k in range(100))),
                          scales=((1.0,) * 100, (0.5,) * 100)),
    "f32": dict(dtype="f32", D=64, Ks=(48, 32), lengths=(40, 50), seg_adapter=(0, 1),
                ranks=((4, 8), (8, 2)), scales=((4.0, 2.0), (2.0, 8.0))),
    "single": dict(dtype="bf16", D=64, Ks=(64,), lengths=(40,), seg_adapter=(0,), ranks=((8,),), scales=((2.0,),)),
}


def run_group(case, w_layouts, save_h, want_w, want_dx, seed=3):
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    c = CASES[case]
    lins, tens = make_group(c["dtype"], c["D"], c["Ks"], c["lengths"], c["seg_adapter"], c["ranks"], c["scales"], seed)
    n = len(lins)
    dps = [gh.upload(lins[p], tens[p], w_layouts[p]) for p in range(n)]
    group = plora.Group([dp.desc for dp in dps])
    ws_bytes = plora.plora_group_workspace_bytes(group)
    assert ws_bytes >= sum(plora.plora_workspace_bytes(dp.desc) for dp in dps)
    guards: list = []
    ws = gh.guarded((ws_bytes,), torch.uint8, None, guards, "group workspace")
    x = dps[0].x
    h = [dps[p].h if save_h[p] else None for p in range(n)]
    plora.plora_group_fwd(group, x, [dp.W for dp in dps], [dp.A for dp in dps], [dp.B for dp in dps], [dp.y for dp in dps],
                          h if any(save_h) else None, ws)
    plora.plora_group_bwd(group, x, [dp.W for dp in dps], [dp.A for dp in dps], [dp.B for dp in dps], [dp.dy for dp in dps],
                          h if any(save_h) else None,
                          [dps[p].dx if want_dx[p] else None for p in range(n)] if any(want_dx) else None,
                          [dps[p].dA if want_w[p] else None for p in range(n)] if any(want_w) else None,
                          [dps[p].dB if want_w[p] else None for p in range(n)] if any(want_w) else None, ws)
    torch.cuda.synchronize()
    for dp in dps:
        gh.check_guards(dp)
    for name, base, nbytes in guards:
        assert bool((base[:gh.GUARD_BYTES] == gh.GUARD_BYTE).all()) and bool((base[gh.GUARD_BYTES + nbytes:] == gh.GUARD_BYTE).all()), name
    return lins, tens, dps


def check_against_oracle(lins, tens, dps, save_h, want_w, want_dx):
    import gpu_harness as gh
    for p, (lin, t, dp) in enumerate(zip(lins, tens, dps)):
        lay = lin.layout
        tol = TOL[lin.dtype]
        prob = make_problem(oracle, lin, t)
        y_o, h_o = oracle.loops.forward(prob)
        dx_o, _, dA_o, dB_o = oracle.loops.backward(prob, t.dy)
        errs = {"y": scaled_err(gh.to_np(dp.y), y_o)}
        if want_dx[p]:
            errs["dx"] = scaled_err(gh.to_np(dp.dx), dx_o)
        else:
            assert bool(dp.dx.float().isnan().all()), f"projection {p}: dx written although not asked for"
        if save_h[p] and lay.sum_Lr() > 0:
            errs["h"] = scaled_err(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)[:lay.sum_Lr()]), h_o)
        for k in range(lay.n_adapters):
            if want_w[p]:
                errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o[k])
                errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o[k])
            else:
                assert bool(dp.dA[k].isnan().all()) and bool(dp.dB[k].isnan().all()), f"projection {p}: gradients written"
        for k, v in errs.items():
            assert np.isfinite(v) and v <= tol, (lin.name, p, k, v, tol)


@pytest.mark.parametrize("case", list(CASES))
@pytest.mark.parametrize("save_h", [True, False])
def test_group_equals_each_projection_alone(case, save_h):
    n = len(CASES[case]["Ks"])
    print(f"[case] group {case} save_h={save_h}", flush=True)
    sys.stdout.flush()
    layouts = [(p + 1) % 2 if case in ("qkv_one_pass", "four") else 0 for p in range(n)]
    sh, ww, wd = [save_h] * n, [True] * n, [True] * n
    lins, tens, dps = run_group(case, layouts, sh, ww, wd)
    check_against_oracle(lins, tens, dps, sh, ww, wd)


@pytest.mark.parametrize("case", ["qkv_one_pass", "cut_in_two", "four"])
def test_group_per_projection_options(case):
    """Saved activation for some projections only, weight gradients for some only, dx for some only: the fused passes
    take the projections that need them, the others run alone or not at all."""
    n = len(CASES[case]["Ks"])
    print(f"[case] group options {case}", flush=True)
    sys.stdout.flush()
    sh = [p % 2 == 0 for p in range(n)]
    ww = [p != 1 for p in range(n)]
    wd = [p != 0 for p in range(n)]
    lins, tens, dps = run_group(case, [0] * n, sh, ww, wd)
    check_against_oracle(lins, tens, dps, sh, ww, wd)


@pytest.mark.parametrize("case", ["qkv_one_pass", "gate_up"])
def test_group_forward_is_bitwise_the_plain_call(case):
    """The fused shrink sums every element over the contraction in the same order as the plain kernel (same stages,
    same splits), so the saved activation and y are bit for bit those of plora_linear_fwd."""
    import torch
    import gpu_harness as gh
    n = len(CASES[case]["Ks"])
    print(f"[case] group bitwise {case}", flush=True)
    sys.stdout.flush()
    lins, tens, dps = run_group(case, [0] * n, [True] * n, [True] * n, [True] * n)
    for p in range(n):
        ref = gh.upload(lins[p], tens[p], 0)
        gh.forward(ref, save_h=True)
        torch.cuda.synchronize()
        nh = lins[p].layout.sum_Lr()
        assert torch.equal(ref.h[:nh], dps[p].h[:nh]), f"projection {p}: saved activation differs"
        assert torch.equal(ref.y, dps[p].y), f"projection {p}: y differs"


@pytest.mark.parametrize("members", [(0, 1, 2), (4, 5)], ids=["q_k_v", "gate_up"])
def test_config4_groups_full_size(members):
    """The decoder layer's two groups at full size (16384 tokens, 16 adapters; q / k / v differ in width): every
    element of h, dA_k and dB_k of every projection against the oracle, and y, dx and h bit for bit against the plain
    calls on the same inputs (whose full-size parity has its own test)."""
    import torch
    import gpu_harness as gh
    import fullsize_checks as fc
    from paper_2508_02932_amd import plora
    lins = [wl.config(4)[i] for i in members]
    print(f"[case] config 4 group {[l.name for l in lins]}", flush=True)
    sys.stdout.flush()
    tens = [l.tensors() for l in lins]
    for t in tens[1:]:
        t.x = tens[0].x
    dps = [gh.upload(l, t, 0) for l, t in zip(lins, tens)]
    group = plora.Group([dp.desc for dp in dps])
    ws = torch.empty(plora.plora_group_workspace_bytes(group), dtype=torch.uint8, device="cuda")
    x = dps[0].x
    plora.plora_group_fwd(group, x, [dp.W for dp in dps], [dp.A for dp in dps], [dp.B for dp in dps], [dp.y for dp in dps],
                          [dp.h for dp in dps], ws)
    plora.plora_group_bwd(group, x, [dp.W for dp in dps], [dp.A for dp in dps], [dp.B for dp in dps], [dp.dy for dp in dps],
                          None, [dp.dx for dp in dps], [dp.dA for dp in dps], [dp.dB for dp in dps], ws)
    torch.cuda.synchronize()
    for p, (lin, t, dp) in enumerate(zip(lins, tens, dps)):
        gh.check_guards(dp)
        lay = lin.layout
        prob = make_problem(oracle, lin, t)
        h_o = oracle.matmul.low_rank_activation(prob)
        dA_o, dB_o = oracle.matmul.low_rank_gradients(prob, t.dy)
        errs = {"h": fc.compare(gh.ragged_h_to_rows(lin, gh.to_np(dp.h)), h_o)}
        for k in range(lay.n_adapters):
            errs[f"dA{k}"] = fc.compare(gh.to_np(dp.dA[k]), dA_o[k])
            errs[f"dB{k}"] = fc.compare(gh.to_np(dp.dB[k]), dB_o[k])
        worst = max(errs.values())
        print(f"  {lin.name}: max error over {len(errs)} tensors {worst:.2e}", flush=True)
        assert all(np.isfinite(v) and v <= TOL["bf16"] for v in errs.values()), (lin.name, errs)
        ref = gh.upload(lin, t, 0)
        gh.forward(ref)
        gh.backward(ref, use_saved_h=False)
        torch.cuda.synchronize()
        nh = lay.sum_Lr()
        assert torch.equal(ref.h[:nh], dp.h[:nh]) and torch.equal(ref.y, dp.y) and torch.equal(ref.dx, dp.dx), lin.name
        del ref
        torch.cuda.empty_cache()
    # the summed input gradient at full size: the chain of bf16 additions of the per-projection results, bit for bit
    chain = dps[0].dx.clone()
    for dp in dps[1:]:
        chain = chain + dp.dx
    dx_sum = torch.full_like(chain, float("nan"))
    plora.plora_group_bwd(group, x, [dp.W for dp in dps], [dp.A for dp in dps], [dp.B for dp in dps], [dp.dy for dp in dps],
                          [dp.h for dp in dps], None, None, None, ws, dx_sum=dx_sum)
    torch.cuda.synchronize()
    assert torch.equal(dx_sum, chain)


@pytest.mark.parametrize("case", ["qkv_one_pass", "cut_in_two", "four", "gate_up", "f32", "single"])
def test_group_input_gradient_summed_in_the_epilogue(case):
    """dx_sum: the gradient of the shared input, sum over the projections of dy_p W_p^T + g_p A_p^T, against the oracle's
    per-projection dx added up in fp64; in bf16 also bit for bit against the chain of bf16 additions of the per-projection
    results (what the accumulating epilogue is specified to equal).  The per-projection dx buffers stay untouched."""
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    c = CASES[case]
    n = len(c["Ks"])
    print(f"[case] group dx_sum {case}", flush=True)
    sys.stdout.flush()
    layouts = [p % 2 for p in range(n)]
    lins, tens, dps = run_group(case, layouts, [True] * n, [True] * n, [True] * n)      # per-projection dx for the chain
    group = plora.Group([dp.desc for dp in dps])
    guards: list = []
    ws = gh.guarded((plora.plora_group_workspace_bytes(group),), torch.uint8, None, guards, "group workspace")
    dx_sum = gh.guarded(tuple(dps[0].dx.shape), dps[0].dx.dtype, float("nan"), guards, "dx_sum")
    chain = dps[0].dx.clone()
    for dp in dps[1:]:
        chain = chain + dp.dx
    for dp in dps:
        dp.dx.fill_(float("nan"))
    lists = lambda name: [getattr(dp, name) for dp in dps]
    plora.plora_group_bwd(group, dps[0].x, lists("W"), lists("A"), lists("B"), lists("dy"), lists("h"), None, lists("dA"), lists("dB"),
                          ws, dx_sum=dx_sum)
    torch.cuda.synchronize()
    for name, base, nbytes in guards:
        assert bool((base[:gh.GUARD_BYTES] == gh.GUARD_BYTE).all()) and bool((base[gh.GUARD_BYTES + nbytes:] == gh.GUARD_BYTE).all()), name
    want = np.zeros(dps[0].dx.shape, dtype=np.float64)
    for lin, t, dp in zip(lins, tens, dps):
        gh.check_guards(dp)
        assert bool(dp.dx.float().isnan().all()), "a per-projection dx was written"
        want += oracle.loops.backward(make_problem(oracle, lin, t), t.dy)[0]
    err = scaled_err(gh.to_np(dx_sum), want)
    assert np.isfinite(err) and err <= TOL[c["dtype"]], (case, err)
    if c["dtype"] == "bf16":
        assert torch.equal(dx_sum, chain), "dx_sum is not the chain of bf16 additions of the per-projection results"
