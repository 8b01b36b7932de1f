"""GPU parity with the frozen weight stored [d_out][d_in] (desc.w_layout = PLORA_W_OUT_IN, the layout of a
framework's linear module).  The layer is the same function of the same matrices (section 2.4, appendix
C.2), so the oracle and the tolerances are those of the other layout; what changes is which form of the
base GEMM runs forward and backward and which packed low-rank operand each reads."""
import numpy as np
import pytest

import oracle
from paper_2508_02932_amd import plora
from paper_2508_02932_amd import workloads as wl
from test_gpu_parity import run_and_compare, _device_tables_equal_export, say

pytestmark = pytest.mark.gpu

OUT_IN = plora.PLORA_W_OUT_IN


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_small_out_in(dtype):
    lin = wl.small(f"ragged_oi_{dtype}", dtype, 328, 264, lengths=[130, 0, 257, 64, 249, 1],
                   seg_adapter=[1, 0, 2, -1, 1, 0], ranks=[8, 24, 72], scales=[2.0, 0.5, 1.25], seed=241)
    run_and_compare(lin, w_layout=OUT_IN)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recompute_h_path_out_in(dtype):
    lin = wl.small(f"recompute_oi_{dtype}", dtype, 256, 192, lengths=[100, 300], seg_adapter=[0, 1],
                   ranks=[16, 40], scales=[2.0, 2.0], seed=243)
    run_and_compare(lin, save_h=False, w_layout=OUT_IN)


def test_several_tiles_out_in():
    """Several 256 x 256 tiles in both directions with d_in != d_out, tiles that straddle more than two segments
    (the walk over the segment table), rank 1, odd rank and the maximum rank."""
    lin = wl.small("tiles_oi", "bf16", 576, 776, lengths=[200, 90, 310, 7, 30, 25, 180],
                   seg_adapter=[0, 1, 2, 3, 1, 2, 0], ranks=[128, 1, 33, 64], scales=[2.0, 4.0, 0.25, 1.0], seed=247)
    run_and_compare(lin, w_layout=OUT_IN)


def test_pure_lora_delta_out_in():
    """W = 0 isolates the low-rank operands of this layout (B_k^T padded in forward, packed A_k^T in backward)."""
    lin = wl.small("w0_oi", "bf16", 512, 264, lengths=[300, 212], seg_adapter=[1, 0], ranks=[16, 72],
                   scales=[2.0, 2.0], seed=253)
    t = lin.tensors()
    t.W = np.zeros_like(t.W)
    run_and_compare(lin, t, w_layout=OUT_IN)


def test_edge_cases_out_in():
    lin = wl.small("edge_oi", "bf16", 64, 72, lengths=[1, 0, 5], seg_adapter=[0, 1, -1], ranks=[4, 16],
                   scales=[1.0, 3.0], seed=261)
    run_and_compare(lin, w_layout=OUT_IN)
    lin = wl.small("base_only_oi", "bf16", 64, 136, lengths=[70], seg_adapter=[-1], ranks=[8], scales=[1.0], seed=267)
    run_and_compare(lin, w_layout=OUT_IN)


def test_device_tables_out_in():
    lin = wl.small("tables_oi", "bf16", 328, 264, lengths=[130, 0, 257, 64, 249, 1, 700, 30, 12],
                   seg_adapter=[1, 0, 2, -1, 1, 0, 3, 2, 0], ranks=[8, 24, 72, 128], scales=[2.0, 0.5, 1.25, 1.0], seed=251)
    _device_tables_equal_export(lin, OUT_IN)


def test_config2_out_in_full():
    """Configuration 2 (4096 x 4096, 8192 tokens) in this layout, every element against the matmul oracle."""
    lin = wl.config(2)[0]
    run_and_compare(lin, impl=oracle.matmul, w_layout=OUT_IN)


def test_unknown_layout_is_refused():
    lin = wl.small("bad_layout", "bf16", 64, 64, lengths=[8], seg_adapter=[0], ranks=[8], scales=[1.0], seed=1)
    lay = lin.layout
    d = plora.Desc(lay.T, lin.D, lin.K, lay.seg_off, lay.seg_adapter, lay.rank, lay.scale, plora.PLORA_BF16, 7)
    assert plora.lib().plora_validate(d.ref) == 8      # PLORA_ERR_UNSUPPORTED
    say("refused")
