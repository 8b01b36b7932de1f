"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle.

The paper prints no numeric example of the packed layer, so every pin is a hand-worked case,
a closed form, an invariant, a special case that reduces to a textbook product, or brute force.
Each pin runs against both writings of the oracle (scalar C loops, numpy matmul).
"""
import itertools
import json
import math
import os

import numpy as np
import pytest

import oracle
from paper_2508_02932_amd import workloads as wl
from util import make_problem, scaled_err

IMPLS = [oracle.loops, oracle.matmul]
IDS = ["loops", "matmul"]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def ragged_case(dtype="f32", seed=3, D=40, K=24):
    """5 segments, repeated adapter, a base-only segment, an empty segment, ranks 1/3/8."""
    lin = wl.small("ragged", dtype, D, K, lengths=[5, 0, 7, 3, 4], seg_adapter=[1, 0, 2, -1, 1],
                   ranks=[3, 8, 1], scales=[0.5, 2.0, 1.25], seed=seed)
    t = lin.tensors()
    return lin, t, make_problem(oracle, lin, t)


# ---------------------------------------------------------------------------------------------
# hand-worked example (tests/golden/hand_worked_rank1.json)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_hand_worked_example(impl):
    with open(os.path.join(GOLDEN, "hand_worked_rank1.json")) as f:
        gold = json.load(f)
    p = oracle.Problem(gold["x"], gold["W"], [np.array(a) for a in gold["A"]],
                       [np.array(b) for b in gold["B"]], gold["seg_off"], gold["seg_adapter"],
                       gold["scale"])
    dy = np.array(gold["dy"], dtype=np.float32)
    y, h = impl.forward(p)
    dx, g, dA, dB = impl.backward(p, dy)
    e = gold["expect"]
    assert np.array_equal(y, np.array(e["y"], dtype=np.float64))
    assert np.array_equal(h[0, :1], np.array(e["h_row0"], dtype=np.float64))
    assert np.array_equal(h[1], np.zeros_like(h[1]))
    assert np.array_equal(g[0, :1], np.array(e["g_row0"], dtype=np.float64))
    assert np.array_equal(dx, np.array(e["dx"], dtype=np.float64))
    assert np.array_equal(dA[0], np.array(e["dA"][0], dtype=np.float64))
    assert np.array_equal(dB[0], np.array(e["dB"][0], dtype=np.float64))


# ---------------------------------------------------------------------------------------------
# brute force on a tiny input: pure-Python sums with math.fsum, written from the definition
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_brute_force_tiny(impl):
    lin = wl.small("tiny", "f32", 6, 5, lengths=[2, 3, 1], seg_adapter=[1, 0, 1], ranks=[2, 3],
                   scales=[0.75, -1.5], seed=11)
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    y, h = impl.forward(p)
    dx, g, dA, dB = impl.backward(p, t.dy)
    T, D, K = p.T, p.D, p.K
    seg_of = []
    for s in range(p.n_seg):
        seg_of += [int(p.seg_adapter[s])] * int(p.seg_off[s + 1] - p.seg_off[s])
    X, W, DY = t.x.astype(float), t.W.astype(float), t.dy.astype(float)
    for tt in range(T):
        k = seg_of[tt]
        r, sc = int(p.rank[k]), float(p.scale[k])
        A, B = t.A[k].astype(float), t.B[k].astype(float)
        hh = [math.fsum(X[tt, i] * A[i, j] for i in range(D)) for j in range(r)]
        gg = [sc * math.fsum(DY[tt, n] * B[j, n] for n in range(K)) for j in range(r)]
        for n in range(K):
            want = math.fsum([X[tt, i] * W[i, n] for i in range(D)]
                             + [sc * hh[j] * B[j, n] for j in range(r)])
            assert abs(y[tt, n] - want) < 1e-13
        for i in range(D):
            want = math.fsum([DY[tt, n] * W[i, n] for n in range(K)]
                             + [gg[j] * A[i, j] for j in range(r)])
            assert abs(dx[tt, i] - want) < 1e-13
        assert np.allclose(h[tt, :r], hh, atol=1e-14) and np.allclose(g[tt, :r], gg, atol=1e-14)
    for k in range(p.n_adapters):
        r, sc = int(p.rank[k]), float(p.scale[k])
        A, B = t.A[k].astype(float), t.B[k].astype(float)
        toks = [tt for tt in range(T) if seg_of[tt] == k]
        for i, j in itertools.product(range(D), range(r)):
            want = math.fsum(X[tt, i] * sc * math.fsum(DY[tt, n] * B[j, n] for n in range(K))
                             for tt in toks)
            assert abs(dA[k][i, j] - want) < 1e-12
        for j, n in itertools.product(range(r), range(K)):
            want = sc * math.fsum(math.fsum(X[tt, i] * A[i, j] for i in range(D)) * DY[tt, n]
                                  for tt in toks)
            assert abs(dB[k][j, n] - want) < 1e-12


# ---------------------------------------------------------------------------------------------
# B = 0: the layer is the base product; dA vanishes (section 2.1: the update is A B)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_zero_B_gives_base_output(impl):
    lin, t, p = ragged_case()
    pz = oracle.Problem(t.x, t.W, t.A, [np.zeros_like(b) for b in t.B], p.seg_off,
                        p.seg_adapter, p.scale)
    base = oracle.Problem(t.x, t.W, [], [], [0, p.T], [-1], [])
    y, _ = impl.forward(pz)
    yb, _ = impl.forward(base)
    assert np.array_equal(y, yb)
    assert np.allclose(yb, t.x.astype(np.float64) @ t.W.astype(np.float64), rtol=0, atol=1e-12)
    dx, g, dA, dB = impl.backward(pz, t.dy)
    dxb, _, _, _ = impl.backward(base, t.dy)
    assert np.array_equal(dx, dxb)
    assert all(np.array_equal(a, np.zeros_like(a)) for a in dA)
    assert np.array_equal(g, np.zeros_like(g))
    # dB does not depend on B: same as with the real B
    _, _, _, dB_real = impl.backward(p, t.dy)
    for a, b in zip(dB, dB_real):
        assert np.array_equal(a, b)


# ---------------------------------------------------------------------------------------------
# packed == each adapter alone (section 2.4: per-adapter computation is ordinary LoRA)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_packed_equals_each_adapter_alone(impl):
    lin, t, p = ragged_case(seed=5)
    y, h = impl.forward(p)
    dx, g, dA, dB = impl.backward(p, t.dy)
    for k in range(p.n_adapters):
        rows = p.rows_of_adapter(k)
        alone = oracle.Problem(t.x[rows], t.W, [t.A[k]], [t.B[k]], [0, len(rows)], [0],
                               [p.scale[k]])
        ya, ha = impl.forward(alone)
        dxa, ga, dAa, dBa = impl.backward(alone, t.dy[rows])
        r = int(p.rank[k])
        if impl is oracle.loops:      # same loops, same order: bit-for-bit
            assert np.array_equal(y[rows], ya) and np.array_equal(dx[rows], dxa)
            assert np.array_equal(h[rows, :r], ha) and np.array_equal(g[rows, :r], ga)
            assert np.array_equal(dA[k], dAa[0]) and np.array_equal(dB[k], dBa[0])
        else:                         # matmul sums segments separately: rounding order differs
            assert np.allclose(y[rows], ya, rtol=0, atol=1e-12)
            assert np.allclose(dx[rows], dxa, rtol=0, atol=1e-12)
            assert np.allclose(dA[k], dAa[0], rtol=0, atol=1e-11)
            assert np.allclose(dB[k], dBa[0], rtol=0, atol=1e-11)


# ---------------------------------------------------------------------------------------------
# merged-weight identity (section 2.1): rows of adapter k equal x (W + scale_k A_k B_k)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_merged_weight_identity(impl):
    lin, t, p = ragged_case(seed=9, D=64, K=48)
    y, _ = impl.forward(p)
    dx, _, _, _ = impl.backward(p, t.dy)
    x64, W64, dy64 = (a.astype(np.float64) for a in (t.x, t.W, t.dy))
    for s in range(p.n_seg):
        k = int(p.seg_adapter[s])
        lo, hi = int(p.seg_off[s]), int(p.seg_off[s + 1])
        Wm = W64 if k < 0 else W64 + float(p.scale[k]) * (
            t.A[k].astype(np.float64) @ t.B[k].astype(np.float64))
        assert np.allclose(y[lo:hi], x64[lo:hi] @ Wm, rtol=0, atol=1e-12)
        assert np.allclose(dx[lo:hi], dy64[lo:hi] @ Wm.T, rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# rank-1 closed form: everything reduces to dot products
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_rank_one_closed_form(impl):
    lin = wl.small("rank1", "f32", 32, 20, lengths=[9], seg_adapter=[0], ranks=[1],
                   scales=[1.75], seed=21)
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    y, h = impl.forward(p)
    dx, g, dA, dB = impl.backward(p, t.dy)
    x, W, dy = (v.astype(np.float64) for v in (t.x, t.W, t.dy))
    a = t.A[0].astype(np.float64)[:, 0]
    b = t.B[0].astype(np.float64)[0, :]
    s = 1.75
    xa = x @ a                      # (x_t . a)
    dyb = dy @ b                    # (dy_t . b)
    assert np.allclose(y, x @ W + s * np.outer(xa, b), rtol=0, atol=1e-12)
    assert np.allclose(dx, dy @ W.T + s * np.outer(dyb, a), rtol=0, atol=1e-12)
    assert np.allclose(dA[0][:, 0], s * (x.T @ dyb), rtol=0, atol=1e-12)
    assert np.allclose(dB[0][0, :], s * (xa @ dy), rtol=0, atol=1e-12)
    assert np.allclose(h[:, 0], xa, rtol=0, atol=1e-13)
    assert np.allclose(g[:, 0], s * dyb, rtol=0, atol=1e-13)


# ---------------------------------------------------------------------------------------------
# central finite differences of L = <y, dy>; L is linear in x, in A_k and in B_k separately, so
# the central difference is exact up to rounding for any step
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_finite_differences(impl):
    lin, t, p = ragged_case(seed=13, D=12, K=10)
    dy64 = t.dy.astype(np.float64)
    dx, g, dA, dB = impl.backward(p, t.dy)
    eps = 2.0 ** -6      # the perturbed float32 values may round: divide by the step actually taken

    def loss(x, A, B):
        q = oracle.Problem(x, t.W, A, B, p.seg_off, p.seg_adapter, p.scale)
        y, _ = impl.forward(q)
        return float(np.sum(y * dy64))

    rng = np.random.default_rng(0)
    for _ in range(25):                 # dX
        tt, i = int(rng.integers(p.T)), int(rng.integers(p.D))
        xp, xm = t.x.copy(), t.x.copy()
        xp[tt, i] += eps
        xm[tt, i] -= eps
        fd = (loss(xp, t.A, t.B) - loss(xm, t.A, t.B)) / (float(xp[tt, i]) - float(xm[tt, i]))
        assert abs(fd - dx[tt, i]) < 1e-9
    for k in range(p.n_adapters):
        r = int(p.rank[k])
        for _ in range(12):             # dA_k
            i, j = int(rng.integers(p.D)), int(rng.integers(r))
            Ap = [a.copy() for a in t.A]
            Am = [a.copy() for a in t.A]
            Ap[k][i, j] += eps
            Am[k][i, j] -= eps
            fd = (loss(t.x, Ap, t.B) - loss(t.x, Am, t.B)) / (float(Ap[k][i, j]) - float(Am[k][i, j]))
            assert abs(fd - dA[k][i, j]) < 1e-9
        for _ in range(12):             # dB_k
            j, n = int(rng.integers(r)), int(rng.integers(p.K))
            Bp = [b.copy() for b in t.B]
            Bm = [b.copy() for b in t.B]
            Bp[k][j, n] += eps
            Bm[k][j, n] -= eps
            fd = (loss(t.x, t.A, Bp) - loss(t.x, t.A, Bm)) / (float(Bp[k][j, n]) - float(Bm[k][j, n]))
            assert abs(fd - dB[k][j, n]) < 1e-9


# ---------------------------------------------------------------------------------------------
# exact small-integer inputs: every product and partial sum is an integer (or a dyadic
# rational), so fp64 must reproduce integer arithmetic exactly
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_exact_integer_inputs(impl):
    rng = np.random.default_rng(42)
    T, D, K = 23, 16, 12
    ranks = [2, 5]
    seg_off, seg_ad = [0, 8, 8, 17, 23], [1, 0, 0, -1]
    x = rng.integers(-2, 3, size=(T, D))
    W = rng.integers(-2, 3, size=(D, K))
    dy = rng.integers(-2, 3, size=(T, K))
    A = [rng.integers(-2, 3, size=(D, r)) for r in ranks]
    B = [rng.integers(-2, 3, size=(r, K)) for r in ranks]
    scale = [2, 4]
    p = oracle.Problem(x, W, A, B, seg_off, seg_ad, scale)
    y, _ = impl.forward(p)
    dx, _, dA, dB = impl.backward(p, dy.astype(np.float32))
    yi = x @ W
    dxi = dy @ W.T
    dAi = [np.zeros((D, r), dtype=np.int64) for r in ranks]
    dBi = [np.zeros((r, K), dtype=np.int64) for r in ranks]
    for s, k in enumerate(seg_ad):
        lo, hi = seg_off[s], seg_off[s + 1]
        if k < 0:
            continue
        yi[lo:hi] += scale[k] * ((x[lo:hi] @ A[k]) @ B[k])
        gi = scale[k] * (dy[lo:hi] @ B[k].T)
        dxi[lo:hi] += gi @ A[k].T
        dAi[k] += x[lo:hi].T @ gi
        dBi[k] += scale[k] * ((x[lo:hi] @ A[k]).T @ dy[lo:hi])
    assert np.array_equal(y, yi.astype(np.float64))
    assert np.array_equal(dx, dxi.astype(np.float64))
    for k in range(2):
        assert np.array_equal(dA[k], dAi[k].astype(np.float64))
        assert np.array_equal(dB[k], dBi[k].astype(np.float64))


# ---------------------------------------------------------------------------------------------
# zero-padding the rank changes nothing (heterogeneous ranks are a bookkeeping matter)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_zero_padded_rank(impl):
    lin, t, p = ragged_case(seed=17)
    pad = 4
    Ap = [np.concatenate([a, np.zeros((p.D, pad), np.float32)], axis=1) for a in t.A]
    Bp = [np.concatenate([b, np.zeros((pad, p.K), np.float32)], axis=0) for b in t.B]
    q = oracle.Problem(t.x, t.W, Ap, Bp, p.seg_off, p.seg_adapter, p.scale)
    y, _ = impl.forward(p)
    yq, _ = impl.forward(q)
    dx, _, dA, dB = impl.backward(p, t.dy)
    dxq, _, dAq, dBq = impl.backward(q, t.dy)
    # the C loops add exact zeros; a BLAS product may group its sums differently when the
    # inner dimension grows, so the matmul writing is compared to rounding only
    same = np.array_equal if impl is oracle.loops else (
        lambda a, b: np.allclose(a, b, rtol=0, atol=1e-12))
    assert same(y, yq) and same(dx, dxq)
    for k in range(p.n_adapters):
        r = int(p.rank[k])
        assert same(dAq[k][:, :r], dA[k]) and same(dBq[k][:r], dB[k])
        # gradient of the padding: columns of A see g = 0, rows of B see h = 0
        assert np.array_equal(dAq[k][:, r:], np.zeros((p.D, pad)))
        assert np.array_equal(dBq[k][r:], np.zeros((pad, p.K)))


# ---------------------------------------------------------------------------------------------
# scale plumbing, permutation of segments, empty adapter, base-only rows
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_scale_times_two_equals_B_times_two(impl):
    lin, t, p = ragged_case(seed=19)
    q1 = oracle.Problem(t.x, t.W, t.A, t.B, p.seg_off, p.seg_adapter, 2 * p.scale)
    q2 = oracle.Problem(t.x, t.W, t.A, [2 * b for b in t.B], p.seg_off, p.seg_adapter, p.scale)
    y1, _ = impl.forward(q1)
    y2, _ = impl.forward(q2)
    assert np.array_equal(y1, y2)
    dx1, _, dA1, dB1 = impl.backward(q1, t.dy)
    dx2, _, dA2, dB2 = impl.backward(q2, t.dy)
    assert np.array_equal(dx1, dx2)
    for k in range(p.n_adapters):
        assert np.array_equal(dA1[k], dA2[k])
        # d/dB of (2s) h B is twice d/d(2B) of s h (2B)
        assert np.array_equal(dB1[k], 2 * dB2[k])


@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_segment_permutation(impl):
    lin, t, p = ragged_case(seed=23)
    order = [3, 0, 4, 2, 1]
    rows = np.concatenate([np.arange(p.seg_off[s], p.seg_off[s + 1]) for s in order]).astype(int)
    lens = [int(p.seg_off[s + 1] - p.seg_off[s]) for s in order]
    off = np.concatenate([[0], np.cumsum(lens)])
    q = oracle.Problem(t.x[rows], t.W, t.A, t.B, off, p.seg_adapter[order], p.scale)
    y, _ = impl.forward(p)
    yq, _ = impl.forward(q)
    dx, _, dA, dB = impl.backward(p, t.dy)
    dxq, _, dAq, dBq = impl.backward(q, t.dy[rows])
    assert np.allclose(yq, y[rows], rtol=0, atol=1e-13)
    assert np.allclose(dxq, dx[rows], rtol=0, atol=1e-13)
    for k in range(p.n_adapters):
        assert np.allclose(dAq[k], dA[k], rtol=0, atol=1e-11)
        assert np.allclose(dBq[k], dB[k], rtol=0, atol=1e-11)


@pytest.mark.parametrize("impl", IMPLS, ids=IDS)
def test_adapter_without_tokens_and_base_only_rows(impl):
    lin = wl.small("edge", "f32", 16, 8, lengths=[4, 0, 6], seg_adapter=[0, 1, -1], ranks=[2, 4],
                   scales=[1.0, 3.0], seed=29)
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    y, h = impl.forward(p)
    dx, g, dA, dB = impl.backward(p, t.dy)
    assert np.array_equal(dA[1], np.zeros((16, 4))) and np.array_equal(dB[1], np.zeros((4, 8)))
    x64, W64, dy64 = (v.astype(np.float64) for v in (t.x, t.W, t.dy))
    assert np.allclose(y[4:], x64[4:] @ W64, rtol=0, atol=1e-13)
    assert np.allclose(dx[4:], dy64[4:] @ W64.T, rtol=0, atol=1e-13)
    assert np.array_equal(h[4:], np.zeros_like(h[4:])) and np.array_equal(g[4:], np.zeros_like(g[4:]))


def test_empty_batch():
    p = oracle.Problem(np.zeros((0, 8)), np.ones((8, 4)), [np.ones((8, 2))], [np.ones((2, 4))],
                       [0, 0], [0], [1.0])
    for impl in IMPLS:
        y, _ = impl.forward(p)
        assert y.shape == (0, 4)
        dx, _, dA, dB = impl.backward(p, np.zeros((0, 4), np.float32))
        assert dx.shape == (0, 8) and not dA[0].any() and not dB[0].any()


# ---------------------------------------------------------------------------------------------
# the two writings agree on a mid-size ragged case; sampled rows equal the full computation
# ---------------------------------------------------------------------------------------------
def test_loops_and_matmul_agree_bf16_inputs():
    lin = wl.small("mid", "bf16", 192, 160, lengths=[70, 33, 130, 1, 64],
                   seg_adapter=[2, 0, 1, -1, 2], ranks=[8, 24, 64], scales=[2.0, 2.0, 0.5], seed=31)
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    y1, h1 = oracle.loops.forward(p)
    y2, h2 = oracle.matmul.forward(p)
    assert scaled_err(y1, y2) < 1e-13 and scaled_err(h1, h2) < 1e-13
    b1 = oracle.loops.backward(p, t.dy)
    b2 = oracle.matmul.backward(p, t.dy)
    assert scaled_err(b1[0], b2[0]) < 1e-13 and scaled_err(b1[1], b2[1]) < 1e-13
    for k in range(p.n_adapters):
        assert scaled_err(b1[2][k], b2[2][k]) < 1e-12
        assert scaled_err(b1[3][k], b2[3][k]) < 1e-12
    rows = np.array([0, 69, 70, 102, 103, 232, 233, 234, 297])
    ys, hs = oracle.loops.fwd_rows(p, rows)
    dxs, gs = oracle.loops.bwd_rows(p, t.dy, rows)
    assert np.array_equal(ys, y1[rows]) and np.array_equal(hs, h1[rows])
    assert np.array_equal(dxs, b1[0][rows]) and np.array_equal(gs, b1[1][rows])


def test_loops_rejects_bad_tables():
    base = dict(x=np.zeros((4, 8)), W=np.zeros((8, 4)), A=[np.zeros((8, 2))], B=[np.zeros((2, 4))],
                scale=[1.0])
    assert oracle.loops.check(oracle.Problem(seg_off=[0, 4], seg_adapter=[0], **base)) == 0
    assert oracle.loops.check(oracle.Problem(seg_off=[0, 3], seg_adapter=[0], **base)) != 0
    assert oracle.loops.check(oracle.Problem(seg_off=[1, 4], seg_adapter=[0], **base)) != 0
    assert oracle.loops.check(oracle.Problem(seg_off=[0, 3, 2, 4], seg_adapter=[0, 0, 0], **base)) != 0
    assert oracle.loops.check(oracle.Problem(seg_off=[0, 4], seg_adapter=[1], **base)) != 0
    assert oracle.loops.check(oracle.Problem(seg_off=[0, 4], seg_adapter=[-2], **base)) != 0


# ---------------------------------------------------------------------------------------------
# the partial entry points used at full size (matmul writing): the activation alone, the weight
# gradients alone, and a subset of the token rows.  Each is pinned by something other than the
# function it abbreviates: pure-Python brute force, finite differences, the hand-worked example,
# and the scalar-loop oracle (itself pinned above).
# ---------------------------------------------------------------------------------------------
def test_low_rank_partials_hand_worked_and_brute_force():
    with open(os.path.join(GOLDEN, "hand_worked_rank1.json")) as f:
        gold = json.load(f)
    p = oracle.Problem(gold["x"], gold["W"], [np.array(a) for a in gold["A"]],
                       [np.array(b) for b in gold["B"]], gold["seg_off"], gold["seg_adapter"],
                       gold["scale"])
    dy = np.array(gold["dy"], dtype=np.float32)
    h = oracle.matmul.low_rank_activation(p)
    dA, dB = oracle.matmul.low_rank_gradients(p, dy)
    e = gold["expect"]
    assert np.array_equal(h[0, :1], np.array(e["h_row0"], dtype=np.float64))
    assert np.array_equal(h[1], np.zeros_like(h[1]))
    assert np.array_equal(dA[0], np.array(e["dA"][0], dtype=np.float64))
    assert np.array_equal(dB[0], np.array(e["dB"][0], dtype=np.float64))
    # brute force (math.fsum over the definition) on a ragged tiny case
    lin = wl.small("tiny2", "f32", 7, 6, lengths=[3, 0, 2, 4], seg_adapter=[1, 0, -1, 1], ranks=[2, 3],
                   scales=[1.5, -0.5], seed=19)
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    h = oracle.matmul.low_rank_activation(p)
    dA, dB = oracle.matmul.low_rank_gradients(p, t.dy)
    X, DY = t.x.astype(float), t.dy.astype(float)
    seg_of = []
    for s in range(p.n_seg):
        seg_of += [int(p.seg_adapter[s])] * int(p.seg_off[s + 1] - p.seg_off[s])
    for tt in range(p.T):
        k = seg_of[tt]
        want = np.zeros(h.shape[1])
        if k >= 0:
            A = t.A[k].astype(float)
            want[:A.shape[1]] = [math.fsum(X[tt, i] * A[i, j] for i in range(p.D)) for j in range(A.shape[1])]
        assert np.allclose(h[tt], want, rtol=0, atol=1e-14)
    for k in range(p.n_adapters):
        r, sc = int(p.rank[k]), float(p.scale[k])
        A, B = t.A[k].astype(float), t.B[k].astype(float)
        toks = [tt for tt in range(p.T) if seg_of[tt] == k]
        for i, j in itertools.product(range(p.D), range(r)):
            want = math.fsum(X[tt, i] * sc * math.fsum(DY[tt, n] * B[j, n] for n in range(p.K)) for tt in toks)
            assert abs(dA[k][i, j] - want) < 1e-12
        for j, n in itertools.product(range(r), range(p.K)):
            want = sc * math.fsum(math.fsum(X[tt, i] * A[i, j] for i in range(p.D)) * DY[tt, n] for tt in toks)
            assert abs(dB[k][j, n] - want) < 1e-12


def test_low_rank_gradients_finite_differences():
    lin, t, p = ragged_case(seed=17, D=12, K=10)
    dy64 = t.dy.astype(np.float64)
    dA, dB = oracle.matmul.low_rank_gradients(p, t.dy)
    eps = 2.0 ** -6

    def loss(A, B):           # through the scalar-loop forward: a different writing of the layer
        y, _ = oracle.loops.forward(oracle.Problem(t.x, t.W, A, B, p.seg_off, p.seg_adapter, p.scale))
        return float(np.sum(y * dy64))

    rng = np.random.default_rng(1)
    for k in range(p.n_adapters):
        r = int(p.rank[k])
        for _ in range(10):
            i, j, n = int(rng.integers(p.D)), int(rng.integers(r)), int(rng.integers(p.K))
            Ap = [a.copy() for a in t.A]
            Am = [a.copy() for a in t.A]
            Ap[k][i, j] += eps
            Am[k][i, j] -= eps
            fd = (loss(Ap, t.B) - loss(Am, t.B)) / (float(Ap[k][i, j]) - float(Am[k][i, j]))
            assert abs(fd - dA[k][i, j]) < 1e-9
            Bp = [b.copy() for b in t.B]
            Bm = [b.copy() for b in t.B]
            Bp[k][j, n] += eps
            Bm[k][j, n] -= eps
            fd = (loss(t.A, Bp) - loss(t.A, Bm)) / (float(Bp[k][j, n]) - float(Bm[k][j, n]))
            assert abs(fd - dB[k][j, n]) < 1e-9


def test_partials_and_row_subsets_equal_scalar_loops():
    lin = wl.small("mid2", "bf16", 136, 120, lengths=[70, 0, 33, 130, 1, 64],
                   seg_adapter=[2, 1, 0, 1, -1, 2], ranks=[8, 24, 64], scales=[2.0, 2.0, 0.5], seed=37)
    t = lin.tensors()
    p = make_problem(oracle, lin, t)
    y1, h1 = oracle.loops.forward(p)
    dx1, g1, dA1, dB1 = oracle.loops.backward(p, t.dy)
    assert scaled_err(oracle.matmul.low_rank_activation(p), h1) < 1e-13
    dA2, dB2 = oracle.matmul.low_rank_gradients(p, t.dy)
    for k in range(p.n_adapters):
        assert scaled_err(dA2[k], dA1[k]) < 1e-12 and scaled_err(dB2[k], dB1[k]) < 1e-12
    # a subset of rows through take_rows: rows next to every segment boundary, a run, the ends
    rows = np.array([0, 1, 69, 70, 71, 102, 103, 104, 150, 151, 152, 153, 232, 233, 234, 297])
    sub = p.take_rows(rows)
    assert sub.T == len(rows) and sub.n_seg == p.n_seg
    for impl in IMPLS:
        ys, hs = impl.forward(sub)
        dxs, gs, _, _ = impl.backward(sub, t.dy[rows])
        assert scaled_err(ys, y1[rows]) < 1e-13 and scaled_err(hs, h1[rows]) < 1e-13
        assert scaled_err(dxs, dx1[rows]) < 1e-13 and scaled_err(gs, g1[rows]) < 1e-13
    ys, _ = oracle.loops.forward(sub)
    assert np.array_equal(ys, oracle.loops.fwd_rows(p, rows)[0])      # the C loops: bit for bit
    assert p.take_rows(np.zeros(0, dtype=np.int64)).T == 0
