"""GPU parity of the NF4 base weight (QLoRA storage; the LoRA computation is unchanged): the expansion kernel bit
for bit against the oracle (an index and a scale decide every value, both sides multiply in fp32 and round once), and
the layer on a stored weight against the oracle's layer on the oracle's expanded values, usual tolerances."""
import numpy as np
import pytest

import oracle
from oracle import nf4
from paper_2508_02932_amd import plora
from paper_2508_02932_amd import workloads as wl
from util import make_problem, scaled_err
from test_gpu_parity import TOL, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n", [64, 64 * 7, 64 * 4099, 4096 * 4096])
def test_dequantize_bit_exact(n, dtype):
    import torch
    say(f"[case] nf4 dequantize n={n} {dtype}")
    codes, absmax = wl.nf4_storage(n, 4096, seed=n % 1000)
    if n >= 64 * 4099:                   # all 256 byte values, every level against large and tiny constants
        codes[:256] = np.arange(256, dtype=np.uint8)
        absmax[:4] = [1.0, 3.0e-5, 1234.5, 0.0]
    want = nf4.dequantize(codes, absmax, n, dtype)
    c = torch.from_numpy(codes).cuda()
    a = torch.from_numpy(absmax).cuda()
    # guard band behind the output
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    out = torch.full((n + 64,), 7.0, dtype=tdt, device="cuda")
    plora.plora_nf4_dequantize(c, a, n, plora.PLORA_BF16 if dtype == "bf16" else plora.PLORA_F32, out)
    torch.cuda.synchronize()
    got = out[:n].float().cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert bool((out[n:] == 7.0).all())


def test_dequantize_bit_exact_at_the_size_of_the_largest_weight():
    """8192 x 28672 weights (configuration 5, mlp_up), the launch bench.py times."""
    test_dequantize_bit_exact(8192 * 28672, "bf16")


def run_nf4_layer(lin, w_layout=0, impl=None):
    import torch
    import gpu_harness as gh
    impl = impl or oracle.loops
    t = lin.tensors()
    tol = TOL[lin.dtype]
    say(f"[case] nf4 layer {lin.name} dtype={lin.dtype} T={lin.layout.T} D={lin.D} K={lin.K} w_layout={w_layout}")
    # the stored weight: W as it lies in memory for this layout, quantised; both sides then use its expanded values
    W_mem = np.ascontiguousarray(t.W.T if w_layout else t.W)
    codes, absmax = nf4.quantize(W_mem.ravel())
    W_deq = nf4.dequantize(codes, absmax, W_mem.size, lin.dtype).reshape(W_mem.shape)
    t.W = np.ascontiguousarray(W_deq.T if w_layout else W_deq)
    p = make_problem(oracle, lin, t)
    y_o, h_o = impl.forward(p)
    dx_o, _, dA_o, dB_o = impl.backward(p, t.dy)

    dp = gh.upload(lin, t, w_layout)
    ws = torch.empty(plora.plora_nf4_workspace_bytes(dp.desc) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:][:plora.plora_nf4_workspace_bytes(dp.desc)]
    c, a = torch.from_numpy(codes).cuda(), torch.from_numpy(absmax).cuda()
    plora.plora_linear_fwd_nf4(dp.desc, dp.x, c, a, dp.A, dp.B, dp.y, dp.h, ws)
    torch.cuda.synchronize()
    plora.plora_linear_bwd_nf4(dp.desc, dp.x, c, a, dp.A, dp.B, dp.dy, dp.h, dp.dx, dp.dA, dp.dB, ws)
    torch.cuda.synchronize()
    gh.check_guards(dp)
    errs = {"y": scaled_err(gh.to_np(dp.y), y_o), "dx": scaled_err(gh.to_np(dp.dx), dx_o)}
    for k in range(lin.layout.n_adapters):
        errs[f"dA{k}"] = scaled_err(gh.to_np(dp.dA[k]), dA_o[k])
        errs[f"dB{k}"] = scaled_err(gh.to_np(dp.dB[k]), dB_o[k])
    say("  errors " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    for k, v in errs.items():
        assert np.isfinite(v) and v <= tol, (lin.name, k, v, tol)


@pytest.mark.parametrize("w_layout", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_nf4_layer_ragged_small(dtype, w_layout):
    lin = wl.small(f"nf4_ragged_{dtype}", dtype, 328, 264, lengths=[130, 0, 257, 64, 249, 1],
                   seg_adapter=[1, 0, 2, -1, 1, 0], ranks=[8, 24, 72], scales=[2.0, 0.5, 1.25], seed=441)
    run_nf4_layer(lin, w_layout)


def test_nf4_layer_config2_full():
    run_nf4_layer(wl.config(2)[0], impl=oracle.matmul)


def test_nf4_errors():
    import torch
    import gpu_harness as gh
    lin = wl.small("nf4_err", "f32", 3, 5, lengths=[4], seg_adapter=[0], ranks=[2], scales=[1.0], seed=1)
    d = gh.desc_of(lin)
    assert plora.plora_nf4_workspace_bytes(d) == 0                 # 15 weights: not a whole number of blocks
    lin = wl.small("nf4_err2", "bf16", 64, 64, lengths=[8], seg_adapter=[0], ranks=[8], scales=[1.0], seed=1)
    dp = gh.upload(lin, lin.tensors())
    codes, absmax = wl.nf4_storage(64 * 64, 64, seed=3)
    c, a = torch.from_numpy(codes).cuda(), torch.from_numpy(absmax).cuda()
    with pytest.raises(plora.PloraError) as e:                     # the ordinary workspace is too small for the expanded weight
        plora.plora_linear_fwd_nf4(dp.desc, dp.x, c, a, dp.A, dp.B, dp.y, None, dp.ws)
    assert e.value.code == 7
    ws = torch.empty(plora.plora_nf4_workspace_bytes(dp.desc), dtype=torch.uint8, device="cuda")
    with pytest.raises(plora.PloraError) as e:
        plora.plora_linear_fwd_nf4(dp.desc, dp.x, None, a, dp.A, dp.B, dp.y, None, ws)
    assert e.value.code == 1
    with pytest.raises(plora.PloraError) as e:
        plora.plora_nf4_dequantize(c, a, 100, plora.PLORA_BF16, ws)
    assert e.value.code == 2
