"""Checks for problems too large for the oracle to compute whole (no layer arithmetic of the
library here; torch is used for sums of products on whichever device the tensors live).

Three parts, used by tests/test_gpu_configs.py on GPU results and by tests/test_fullsize_checks.py
on CPU stand-ins with planted mistakes:

* ``plan_rows``      - which token rows get their y, h, dx computed by the oracle: whole 256-row
                       tiles spread over the batch (first and last included), the rows around every
                       segment boundary and around the boundaries of the first and last 256-row tile
                       of every segment, and seeded random rows.
* ``adjoint_per_row`` - the layer is linear in x and acts on each token row by itself (section 2.4),
                       so for any probe u:  <dy_t, f(u)_t> = <dx_t, u_t>  for EVERY row t, where
                       dx is the backward result for dy (appendix C.2 case 4).  Each row's identity
                       is held to the rounding noise of that row, so one wrong 256-wide piece of
                       one row fails it.
* ``compare``        - scaled element-wise error of a block against the oracle.

Noise model of ``adjoint_per_row``: y_u and dx are rounded to bf16 (8 significant bits) once from
fp32 sums: relative error at most 2^-8 per element, independent between elements, so
    lhs_t - rhs_t  has standard deviation  <=  2^-8 / sqrt(3) * sqrt(S1_t^2 + S2_t^2),
    S1_t^2 = sum_n (dy_tn y_tn)^2,   S2_t^2 = sum_i (dx_ti u_ti)^2.
The bound used is  c * 2^-8 * (S1_t + S2_t)  with c = 3, i.e. at least 5.2 of those standard
deviations and in practice more than 7 (the rounding error of a value inside its binade is smaller
than the worst case; the largest ratio observed on correct results over 10^5 rows is 0.56).  The
rounding of the low-rank factors to bf16 inside the kernels adds a term of the same form that is
smaller by the ratio of the low-rank update to the base product and is covered by the margin.
"""
from __future__ import annotations

import numpy as np
import torch

TILE = 256


def plan_rows(seg_off, n_whole_tiles: int, n_random: int, rng: np.random.Generator, tile: int = TILE) -> np.ndarray:
    seg_off = np.asarray(seg_off, dtype=np.int64)
    T = int(seg_off[-1])
    if T == 0:
        return np.zeros(0, dtype=np.int64)
    rows = set()
    tiles_m = (T + tile - 1) // tile
    # whole tiles, spread evenly with the first and the last one included
    picks = {0, tiles_m - 1} | {int(round(i * (tiles_m - 1) / max(n_whole_tiles - 1, 1))) for i in range(n_whole_tiles)}
    for m in picks:
        rows.update(range(m * tile, min((m + 1) * tile, T)))
    # segment boundaries and the boundaries of the first and last tile of each segment, 2 rows each side
    marks = set()
    for s in range(len(seg_off) - 1):
        lo, hi = int(seg_off[s]), int(seg_off[s + 1])
        if hi == lo:
            continue
        marks.update((lo, hi))
        for edge in (lo, hi - 1):
            marks.update((edge // tile * tile, edge // tile * tile + tile))
    for b in marks:
        rows.update(r for r in range(b - 2, b + 2) if 0 <= r < T)
    rows.update(int(v) for v in rng.integers(0, T, size=n_random))
    return np.array(sorted(rows), dtype=np.int64)


def adjoint_per_row(dy: torch.Tensor, y_u: torch.Tensor, dx: torch.Tensor, u: torch.Tensor, c: float = 3.0,
                    chunk: int = 2048) -> dict:
    """Row-wise adjoint identity with the rounding-noise bound of the module docstring.

    Returns {"n_bad", "bad_rows" (first 16), "worst" (largest |lhs-rhs| / bound)}; NaN or Inf anywhere
    in a row makes that row bad."""
    T = dy.shape[0]
    assert y_u.shape == dy.shape and dx.shape == u.shape and dx.shape[0] == T
    bad_rows, worst, n_bad = [], 0.0, 0
    for t0 in range(0, T, chunk):
        sl = slice(t0, min(t0 + chunk, T))
        p1 = dy[sl].double() * y_u[sl].double()
        p2 = dx[sl].double() * u[sl].double()
        lhs, rhs = p1.sum(1), p2.sum(1)
        bound = c * 2.0 ** -8 * (p1.square().sum(1).sqrt() + p2.square().sum(1).sqrt()) + 1e-30
        ratio = (lhs - rhs).abs() / bound
        ratio = torch.where(torch.isfinite(ratio), ratio, torch.full_like(ratio, float("inf")))
        bad = torch.nonzero(ratio > 1.0).flatten()
        n_bad += int(bad.numel())
        if bad.numel() and len(bad_rows) < 16:
            bad_rows += [t0 + int(b) for b in bad[:16 - len(bad_rows)].tolist()]
        if ratio.numel():
            worst = max(worst, float(ratio.max().item()))
    return {"n_bad": n_bad, "bad_rows": bad_rows, "worst": worst}


def adjoint_global_old(dy, y_u, dx, u) -> float:
    """The normalisation this module replaces, kept only so that the mutation test can show why:
    |<dy, y_u> - <dx, u>| / (||dy|| ||y_u||).  Two unrelated vectors of N elements already give about
    1/sqrt(N), so a bound of 2e-3 passes with dx = 0."""
    lhs = float((dy.double() * y_u.double()).sum())
    rhs = float((dx.double() * u.double()).sum())
    return abs(lhs - rhs) / float(dy.double().norm() * y_u.double().norm())


def compare(got, want) -> float:
    """max_i |got_i - want_i| / (|want_i| + rms(want)); NaN in got counts as infinite."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    if not np.isfinite(got).all():
        return float("inf")
    rms = float(np.sqrt(np.mean(want * want)))
    diff = np.abs(got - want)
    return float(diff.max()) if rms == 0.0 else float((diff / (np.abs(want) + rms)).max())
