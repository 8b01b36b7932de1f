"""The entry point that allocates nothing (plora_linear_fwd_noalloc) against plora_linear_fwd: same
bits, on two calls in a row, the second with a smaller input (the scratch array keeps the first
call's contents)."""
import numpy as np
import pytest

from paper_2508_02932_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_noalloc_forward_equals_forward_twice_in_a_row():
    import torch
    import gpu_harness as gh
    from paper_2508_02932_amd import plora
    big = wl.small("noalloc_big", "bf16", 1024, 1536, lengths=[700, 0, 1290, 258, 301], seg_adapter=[0, 1, 2, -1, 0],
                   ranks=[64, 8, 33], scales=[2.0, 1.0, 0.5], seed=131)
    small = wl.small("noalloc_small", "bf16", 264, 328, lengths=[130, 77], seg_adapter=[1, 0], ranks=[128, 16],
                     scales=[0.5, 2.0], seed=137)
    for lin in (big, small):
        print(f"[case] {lin.name}", flush=True)
        t = lin.tensors()
        ref = gh.upload(lin, t)
        gh.forward(ref)
        torch.cuda.synchronize()
        dp = gh.upload(lin, t)
        assert plora.plora_workspace_bytes(dp.desc) <= plora.NOALLOC_SCRATCH_BYTES
        plora.plora_linear_fwd_noalloc(dp.desc, dp.x, dp.W, dp.A, dp.B, dp.y, dp.h)
        torch.cuda.synchronize()
        gh.check_guards(dp)
        assert np.array_equal(gh.to_np(dp.y), gh.to_np(ref.y))
        assert not np.isnan(gh.to_np(dp.y)).any()
        n = lin.layout.sum_Lr()
        assert np.array_equal(gh.to_np(dp.h)[:n], gh.to_np(ref.h)[:n])
    # a description that needs more than the scratch array holds is refused before any launch
    huge = wl.config(5)[1]
    d = gh.desc_of(huge)
    assert plora.plora_workspace_bytes(d) > plora.NOALLOC_SCRATCH_BYTES
    with pytest.raises(plora.PloraError) as e:
        plora.plora_linear_fwd_noalloc(d, dp.x, dp.W, dp.A, dp.B, dp.y, dp.h)
    assert e.value.code == 7
