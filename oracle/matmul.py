"""The packed multi-LoRA layer written with numpy's fp64 matrix product as the only step.

Test infrastructure only.  Same definition as the scalar-loop oracle (paper sections 2.1 and
2.4, gradient cases 1-4 of appendix C.2), one line per formula, so that whole tensors of the
larger configurations can be checked.  Inputs are widened to fp64 first; nothing is blocked,
fused or reordered beyond "one segment at a time".
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

from .problem import Problem


def forward(p: Problem) -> Tuple[np.ndarray, np.ndarray]:
    """(y[T, K], h[T, r_max]); h is zero beyond each row's rank.

    y_t = x_t W + scale_k (x_t A_k) B_k for the tokens t of adapter k (section 2.1 merged
    form, applied per segment as section 2.4 prescribes)."""
    x = p.x.astype(np.float64)
    W = p.W.astype(np.float64)
    y = x @ W
    pitch = int(p.rank.max()) if p.n_adapters else 1
    h = np.zeros((p.T, pitch), dtype=np.float64)
    for s in range(p.n_seg):
        k = int(p.seg_adapter[s])
        lo, hi = int(p.seg_off[s]), int(p.seg_off[s + 1])
        if k < 0 or hi == lo:
            continue
        r = int(p.rank[k])
        hs = x[lo:hi] @ p.A[k].astype(np.float64)
        h[lo:hi, :r] = hs
        y[lo:hi] += float(p.scale[k]) * (hs @ p.B[k].astype(np.float64))
    return y, h


def backward(p: Problem, dy: np.ndarray
             ) -> Tuple[np.ndarray, np.ndarray, List[np.ndarray], List[np.ndarray]]:
    """(dx[T, D], g[T, r_max], [dA_k], [dB_k]) for upstream gradient dy[T, K]."""
    x = p.x.astype(np.float64)
    W = p.W.astype(np.float64)
    dy = np.asarray(dy, dtype=np.float32).astype(np.float64)
    dx = dy @ W.T                                             # base part of case 4
    pitch = int(p.rank.max()) if p.n_adapters else 1
    g = np.zeros((p.T, pitch), dtype=np.float64)
    dA = [np.zeros((p.D, int(r)), dtype=np.float64) for r in p.rank]
    dB = [np.zeros((int(r), p.K), dtype=np.float64) for r in p.rank]
    for s in range(p.n_seg):
        k = int(p.seg_adapter[s])
        lo, hi = int(p.seg_off[s]), int(p.seg_off[s + 1])
        if k < 0 or hi == lo:
            continue
        r = int(p.rank[k])
        sc = float(p.scale[k])
        Ak = p.A[k].astype(np.float64)
        Bk = p.B[k].astype(np.float64)
        gs = sc * (dy[lo:hi] @ Bk.T)                          # case 2
        g[lo:hi, :r] = gs
        dx[lo:hi] += gs @ Ak.T                                # case 4
        dA[k] += x[lo:hi].T @ gs                              # case 3
        dB[k] += sc * ((x[lo:hi] @ Ak).T @ dy[lo:hi])         # case 1
    return dx, g, dA, dB


def low_rank_activation(p: Problem) -> np.ndarray:
    """h[T, r_max] alone: h_t = x_t A_k for the tokens of adapter k (section 2.4), zero beyond
    each row's rank and for base-only rows.  Same line as in ``forward``, without the base
    product, so that the saved activation of a full-size problem can be checked whole."""
    x = p.x.astype(np.float64)
    pitch = int(p.rank.max()) if p.n_adapters else 1
    h = np.zeros((p.T, pitch), dtype=np.float64)
    for s in range(p.n_seg):
        k = int(p.seg_adapter[s])
        lo, hi = int(p.seg_off[s]), int(p.seg_off[s + 1])
        if k < 0 or hi == lo:
            continue
        h[lo:hi, :int(p.rank[k])] = x[lo:hi] @ p.A[k].astype(np.float64)
    return h


def low_rank_gradients(p: Problem, dy: np.ndarray) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """([dA_k], [dB_k]) alone: gradient cases 1-3 of appendix C.2 without the base product of
    case 4 (dx), so that every adapter's gradients of a full-size problem can be checked.

        g_t  = scale_k dy_t B_k^T                  (case 2)
        dA_k = sum_t x_t^T g_t                     (case 3)
        dB_k = scale_k sum_t (x_t A_k)^T dy_t      (case 1)
    """
    x = p.x.astype(np.float64)
    dy = np.asarray(dy, dtype=np.float32)
    dA = [np.zeros((p.D, int(r)), dtype=np.float64) for r in p.rank]
    dB = [np.zeros((int(r), p.K), dtype=np.float64) for r in p.rank]
    for s in range(p.n_seg):
        k = int(p.seg_adapter[s])
        lo, hi = int(p.seg_off[s]), int(p.seg_off[s + 1])
        if k < 0 or hi == lo:
            continue
        sc = float(p.scale[k])
        Ak = p.A[k].astype(np.float64)
        Bk = p.B[k].astype(np.float64)
        dys = dy[lo:hi].astype(np.float64)
        gs = sc * (dys @ Bk.T)                                # case 2
        dA[k] += x[lo:hi].T @ gs                              # case 3
        dB[k] += sc * ((x[lo:hi] @ Ak).T @ dys)               # case 1
    return dA, dB
