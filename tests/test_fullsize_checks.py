"""Mutation tests of the full-size checkers (CPU only).  The mistakes are planted in stand-ins for
the library's outputs built from the oracle: fp64 results rounded once to bf16, which is what a
correct library returns.  Every planted mistake must turn the per-row adjoint check red, the
unplanted stand-in must stay green, and the normalisation the check replaces is shown not to
notice a result that is identically zero."""
import numpy as np
import pytest
import torch

import oracle
import fullsize_checks as fc
from paper_2508_02932_amd import workloads as wl
from util import make_problem


def bf16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(wl.round_to_bf16(np.asarray(a, dtype=np.float32))).to(torch.bfloat16)


@pytest.fixture(scope="module")
def case():
    lin = wl.small("mut", "bf16", 1024, 768, lengths=[300, 212, 0, 515, 253, 256],
                   seg_adapter=[0, 1, 2, -1, 1, 3], ranks=[16, 64, 8, 33], scales=[2.0, 2.0, 1.0, 0.5], seed=211)
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    rng = np.random.default_rng(5)
    u = wl.round_to_bf16(rng.standard_normal(t.x.shape).astype(np.float32))
    pu = oracle.Problem(u, t.W, t.A, t.B, p.seg_off, p.seg_adapter, p.scale)
    y_u, _ = oracle.matmul.forward(pu)
    dx, g, _, _ = oracle.matmul.backward(p, t.dy)
    return dict(lin=lin, t=t, p=p, u=torch.from_numpy(u).to(torch.bfloat16), y_u=y_u, dx=dx, g=g,
                dy=torch.from_numpy(t.dy).to(torch.bfloat16))


def test_correct_results_pass(case):
    res = fc.adjoint_per_row(case["dy"], bf16(case["y_u"]), bf16(case["dx"]), case["u"])
    assert res["n_bad"] == 0 and res["worst"] < 0.7, res
    # and in the launch shape of the GPU test: chunked over rows
    res = fc.adjoint_per_row(case["dy"], bf16(case["y_u"]), bf16(case["dx"]), case["u"], chunk=100)
    assert res["n_bad"] == 0


def test_zeroed_tile_of_dx_is_caught_and_was_not_before(case):
    dx = case["dx"].copy()
    dx[512:768, 256:512] = 0.0                    # one 256 x 256 output tile never written
    res = fc.adjoint_per_row(case["dy"], bf16(case["y_u"]), bf16(dx), case["u"])
    assert res["n_bad"] >= 200 and all(512 <= r < 768 for r in res["bad_rows"]), res
    # the normalisation used before: even dx = 0 everywhere stays far below its 2e-3 bound
    assert fc.adjoint_global_old(case["dy"], bf16(case["y_u"]), bf16(dx), case["u"]) < 2e-3
    assert fc.adjoint_global_old(case["dy"], bf16(case["y_u"]), bf16(0 * dx), case["u"]) < 2e-3
    res0 = fc.adjoint_per_row(case["dy"], bf16(case["y_u"]), bf16(0 * dx), case["u"])
    assert res0["n_bad"] > 0.9 * dx.shape[0]


def test_zeroed_tile_of_y_is_caught(case):
    y = case["y_u"].copy()
    y[1280:1536, 512:768] = 0.0
    res = fc.adjoint_per_row(case["dy"], bf16(y), bf16(case["dx"]), case["u"])
    assert res["n_bad"] >= 200 and all(1280 <= r < 1536 for r in res["bad_rows"]), res


def test_dropped_contraction_stage_is_caught(case):
    """One 64-deep step of the contraction left out of one tile of dx (dx = dy W^T + ...: the step is
    64 columns of dy against 64 columns of W)."""
    t = case["t"]
    dx = case["dx"].copy()
    dx[0:256, 0:256] -= t.dy[0:256, 128:192].astype(np.float64) @ t.W[0:256, 128:192].astype(np.float64).T
    res = fc.adjoint_per_row(case["dy"], bf16(case["y_u"]), bf16(dx), case["u"])
    assert res["n_bad"] >= 100 and all(r < 256 for r in res["bad_rows"]), res


def test_wrong_adapter_in_backward_is_caught(case):
    """Rows 300..511 (adapter 1) get the low-rank term of adapter 3 in dx only."""
    t, p = case["t"], case["p"]
    lay = case["lin"].layout
    wrong = lay.seg_adapter.copy()
    wrong[1] = 3
    pw = oracle.Problem(t.x, t.W, t.A, t.B, p.seg_off, wrong, p.scale)
    dxw, _, _, _ = oracle.matmul.backward(pw, t.dy)
    res = fc.adjoint_per_row(case["dy"], bf16(case["y_u"]), bf16(dxw), case["u"])
    assert res["n_bad"] >= 150 and all(300 <= r < 512 for r in res["bad_rows"]), res


def test_nan_rows_are_bad(case):
    dx = bf16(case["dx"]).clone()
    dx[7, 3] = float("nan")
    res = fc.adjoint_per_row(case["dy"], bf16(case["y_u"]), dx, case["u"])
    assert res["n_bad"] == 1 and res["bad_rows"] == [7]


def test_compare_flags_a_zeroed_tile_and_nan(case):
    y = wl.round_to_bf16(case["y_u"].astype(np.float32)).astype(np.float64)
    assert fc.compare(y, case["y_u"]) < 1e-2
    y2 = y.copy()
    y2[256:512, 0:256] = 0.0
    assert fc.compare(y2, case["y_u"]) > 0.5
    y2 = y.copy()
    y2[1, 1] = np.nan
    assert fc.compare(y2, case["y_u"]) == float("inf")


def test_plan_rows_covers_what_it_promises():
    rng = np.random.default_rng(3)
    seg_off = np.array([0, 700, 700, 1300, 4096, 5000, 9999])
    rows = fc.plan_rows(seg_off, n_whole_tiles=5, n_random=64, rng=rng)
    T = 9999
    assert np.all(np.diff(rows) > 0) and rows[0] == 0 and rows[-1] == T - 1
    have = set(rows.tolist())
    assert set(range(0, 256)) <= have and set(range(9984, T)) <= have        # first and last tile, whole
    n_whole = sum(1 for m in range(T // 256 + 1) if set(range(m * 256, min(m * 256 + 256, T))) <= have)
    assert n_whole >= 5
    for b in (700, 1300, 4096, 5000):                                         # segment boundaries
        assert {b - 2, b - 1, b, b + 1} <= have
    for b in (256, 512, 768, 1280, 1536, 3840, 4352, 4864, 5120, 9984):      # tile boundaries of first / last tiles
        assert {b - 2, b - 1, b, b + 1} <= have, b
    assert len(fc.plan_rows(np.array([0, 0]), 4, 8, rng)) == 0
