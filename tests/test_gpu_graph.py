"""The calls under HIP graph capture: a forward and a backward call recorded once and replayed several times, with
eager work of the same program between the replays, must reproduce the eager results bit for bit every time (the
calls only enqueue kernels - no synchronisation, no memset, no host-side allocation - and the packing description
travels as a kernel argument, so a replay needs nothing from the host)."""
import numpy as np
import pytest

from paper_2508_02932_amd import plora
from paper_2508_02932_amd import workloads as wl
from test_gpu_parity import say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["fused", "lora_only"])
def test_capture_and_replay(mode):
    import torch
    import gpu_harness as gh
    lin = wl.small(f"graph_{mode}", "bf16", 328, 264, lengths=[130, 0, 257, 64, 249, 1, 300],
                   seg_adapter=[1, 0, 2, -1, 1, 0, 2], ranks=[8, 24, 72], scales=[2.0, 0.5, 1.25], seed=541)
    t = lin.tensors()
    lora_only = mode == "lora_only"
    dp = gh.upload(lin, t, lora_only=lora_only)
    base_y = torch.randn_like(dp.y)
    base_dx = torch.randn_like(dp.dx)

    def step():
        if lora_only:
            dp.y.copy_(base_y)
            dp.dx.copy_(base_dx)
            gh.lora_forward(dp)
            gh.lora_backward(dp)
        else:
            gh.forward(dp)
            gh.backward(dp)

    def snapshot():
        torch.cuda.synchronize()
        return [dp.y.clone(), dp.dx.clone(), dp.h.clone()] + [a.clone() for a in dp.dA] + [b.clone() for b in dp.dB]

    step()                                         # eager: also the one-time set-up of the library on this device
    want = snapshot()
    say(f"[case] graph capture {mode}")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                     # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        # eager work of the same program between replays: scribble over the outputs and the workspace
        for buf in (dp.y, dp.dx, dp.h, *dp.dA, *dp.dB):
            buf.fill_(float("nan"))
        dp.ws.fill_(0xAB)
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep} differs from the eager run"
    gh.check_guards(dp)


def test_capture_and_replay_grouped():
    """The grouped calls (three projections on one x, one fused pass each way) under capture: as above."""
    import torch
    import gpu_harness as gh
    lengths, seg_adapter = [130, 0, 257, 64, 249], [1, 0, 2, -1, 1]
    lins = [wl.small(f"graph_group_p{p}", "bf16", 328, K, lengths, seg_adapter, ranks, [2.0, 0.5, 1.25], seed=560 + p)
            for p, (K, ranks) in enumerate(((264, [8, 24, 40]), (64, [16, 16, 33]), (72, [1, 32, 7])))]
    tens = [l.tensors() for l in lins]
    for t in tens[1:]:
        t.x = tens[0].x
    dps = [gh.upload(l, t, p % 2) for p, (l, t) in enumerate(zip(lins, tens))]
    group = plora.Group([dp.desc for dp in dps])
    guards: list = []
    ws = gh.guarded((plora.plora_group_workspace_bytes(group),), torch.uint8, None, guards, "group workspace")
    x = dps[0].x
    lists = lambda name: [getattr(dp, name) for dp in dps]

    def step():
        plora.plora_group_fwd(group, x, lists("W"), lists("A"), lists("B"), lists("y"), lists("h"), ws)
        plora.plora_group_bwd(group, x, lists("W"), lists("A"), lists("B"), lists("dy"), None, lists("dx"), lists("dA"), lists("dB"), ws)

    outputs = lambda: [b for dp in dps for b in (dp.y, dp.dx, dp.h, *dp.dA, *dp.dB)]

    def snapshot():
        torch.cuda.synchronize()
        return [b.clone() for b in outputs()]

    step()
    want = snapshot()
    say("[case] graph capture grouped")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for buf in outputs():
            buf.fill_(float("nan"))
        ws.fill_(0xAB)
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep} differs from the eager run"
    for dp in dps:
        gh.check_guards(dp)
    for name, base, nbytes in guards:
        assert bool((base[:gh.GUARD_BYTES] == gh.GUARD_BYTE).all()) and bool((base[gh.GUARD_BYTES + nbytes:] == gh.GUARD_BYTE).all()), name
