"""Pins of the NF4 oracle (CPU only): the level table against its quantile construction and against the
properties the format is published with, the nibble order and the block scaling on hand-worked bytes, the bf16
rounding against a library conversion, and the quantise / dequantise round trip against its error bound."""
import numpy as np
import pytest
import torch
from scipy.stats import norm

import oracle
from oracle import nf4


def test_table_is_the_quantile_construction():
    built = nf4.table_from_quantiles()
    assert built.shape == (16,)
    # the stored constants were first computed in fp32: agreement to fp32 resolution, not bit for bit
    assert np.abs(built - nf4.TABLE.astype(np.float64)).max() < 2e-7
    # a wrong digit anywhere above the seventh decimal fails the line above; the order of the entries:
    assert np.all(np.diff(nf4.TABLE) > 0)


def test_table_properties_of_the_format():
    t = nf4.TABLE.astype(np.float64)
    assert t[0] == -1.0 and t[15] == 1.0 and t[7] == 0.0            # full range used, zero exact
    assert (t < 0).sum() == 7 and (t > 0).sum() == 8                # one more positive level than negative
    # the levels are normal quantiles: equal probability steps on each side of zero (checked from the CDF side)
    z = norm.ppf(0.9677083)
    p_pos = norm.cdf(t[8:] * z)
    p_neg = norm.cdf(-t[:7] * z)
    assert np.allclose(np.diff(p_pos), np.diff(p_pos)[0], atol=2e-7)
    assert np.allclose(np.diff(p_neg), np.diff(p_neg)[0], atol=2e-7)
    assert abs(np.diff(p_pos)[0] - (0.9677083 - 0.5) / 8) < 2e-7 and abs(-np.diff(p_neg)[0] - (0.9677083 - 0.5) / 7) < 2e-7


def test_storage_cost_is_four_and_a_half_bits_per_weight():
    w = np.random.default_rng(0).standard_normal(64 * 100)
    codes, absmax = nf4.quantize(w)
    assert (codes.nbytes + absmax.nbytes) * 8 == 4.5 * w.size       # 4 bits + one fp32 per 64 elements


def test_hand_worked_bytes():
    # one block: bytes 0x0F 0x7A then 0x88 ...: element 0 = level 0 (-1), element 1 = level 15 (+1), element 2 = level 7
    # (0), element 3 = level 10, the rest level 8; absmax 2 -> values -2, 2, 0, 2 * 0.24611230194568634, 2 * 0.0795802...
    codes = np.array([0x0F, 0x7A] + [0x88] * 30, dtype=np.uint8)
    idx = nf4.unpack(codes, 64)
    assert idx[:4].tolist() == [0, 15, 7, 10] and set(idx[4:].tolist()) == {8}
    v = nf4.dequantize(codes, np.array([2.0], dtype=np.float32), 64, "f32")
    assert v[0] == -2.0 and v[1] == 2.0 and v[2] == 0.0
    assert v[3] == np.float32(0.24611230194568634) * np.float32(2.0)
    assert np.all(v[4:] == np.float32(0.07958029955625534) * np.float32(2.0))
    # second block scales by its own constant
    v2 = nf4.dequantize(np.concatenate([codes, codes]), np.array([2.0, 0.5], dtype=np.float32), 128, "f32")
    assert v2[64] == -0.5 and v2[65] == 0.5 and np.array_equal(v2[:64], v)


def test_bf16_rounding_matches_a_library_conversion():
    rng = np.random.default_rng(1)
    a = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 3,
                        # exact ties between two bf16 neighbours, both parities
                        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.0, 2.0 ** -130], dtype=np.float32)])
    want = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    assert np.array_equal(nf4._round_bf16(a), want)
    codes = rng.integers(0, 256, size=32 * 50, dtype=np.uint8)
    absmax = (rng.random(50).astype(np.float32) + 0.01)
    f = nf4.dequantize(codes, absmax, 64 * 50, "f32")
    b = nf4.dequantize(codes, absmax, 64 * 50, "bf16")
    assert np.array_equal(b, torch.from_numpy(f).to(torch.bfloat16).float().numpy())


def test_round_trip_error_bound_and_exact_levels():
    rng = np.random.default_rng(2)
    w = rng.standard_normal(64 * 200) * 0.02
    codes, absmax = nf4.quantize(w)
    back = nf4.dequantize(codes, absmax, w.size, "f32").astype(np.float64)
    half_gap = np.diff(nf4.TABLE.astype(np.float64)).max() / 2       # nearest level: at most half the widest gap away
    assert np.all(np.abs(back - w) <= np.repeat(absmax, 64) * (half_gap + 1e-6))
    # every block reproduces its largest element (it sits on level +-1)
    blocks_w, blocks_b = w.reshape(-1, 64), back.reshape(-1, 64)
    j = np.abs(blocks_w).argmax(axis=1)
    got = blocks_b[np.arange(len(j)), j]
    assert np.allclose(got, blocks_w[np.arange(len(j)), j], rtol=1e-6)
    # values that are levels times a power of two come back exactly, with the indices they were made from
    idx = rng.integers(0, 16, size=64 * 10).astype(np.uint8)
    idx[::64] = 15                                                   # each block contains its absmax
    exact = nf4.TABLE[idx].astype(np.float64) * 0.25
    c2, a2 = nf4.quantize(exact)
    assert np.array_equal(nf4.unpack(c2, exact.size), idx) and np.all(a2 == 0.25)
    assert np.array_equal(nf4.dequantize(c2, a2, exact.size, "f32").astype(np.float64), exact)


def test_layer_on_a_quantised_weight_is_the_layer_on_its_values():
    """What 'the LoRA computation is unchanged' means for the oracle: nothing but W differs."""
    from paper_2508_02932_amd import workloads as wl
    from util import make_problem
    lin = wl.small("nf4_layer", "bf16", 64, 128, lengths=[20, 12], seg_adapter=[0, 1], ranks=[4, 8], scales=[2.0, 1.0], seed=5)
    t = lin.tensors()
    codes, absmax = nf4.quantize(t.W.ravel())
    t.W = nf4.dequantize(codes, absmax, t.W.size, "bf16").reshape(t.W.shape)
    p = make_problem(oracle, lin, t)
    y, _ = oracle.loops.forward(p)
    want = t.x.astype(np.float64) @ t.W.astype(np.float64)
    for s in range(2):
        lo, hi = int(lin.layout.seg_off[s]), int(lin.layout.seg_off[s + 1])
        k = int(lin.layout.seg_adapter[s])
        want[lo:hi] += float(lin.layout.scale[k]) * (t.x[lo:hi].astype(np.float64) @ t.A[k].astype(np.float64)) @ t.B[k].astype(np.float64)
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)
