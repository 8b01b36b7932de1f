"""Container for one packed multi-LoRA problem as the oracle sees it.  Test infrastructure only.

Notation follows the paper (section 2.1): W in R^{d x k} (here ``D x K``), A_k in R^{d x r_k},
B_k in R^{r_k x k}; tokens are rows of x (row-vector convention); segment s holds rows
``seg_off[s] .. seg_off[s+1]-1`` and belongs to adapter ``seg_adapter[s]`` (-1: base only).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


@dataclass
class Problem:
    x: np.ndarray                 # [T, D]  float32 holding the already-rounded input values
    W: np.ndarray                 # [D, K]
    A: List[np.ndarray]           # A[k]: [D, r_k]
    B: List[np.ndarray]           # B[k]: [r_k, K]
    seg_off: np.ndarray           # [n_seg+1] int32
    seg_adapter: np.ndarray       # [n_seg]   int32
    scale: np.ndarray             # [n_adapters] float32 (alpha_k / r_k, chosen by the caller)
    rank: np.ndarray = field(default=None)  # [n_adapters] int32, derived from A if None

    def __post_init__(self):
        self.x = _f32(self.x)
        self.W = _f32(self.W)
        self.A = [_f32(a) for a in self.A]
        self.B = [_f32(b) for b in self.B]
        self.seg_off = np.ascontiguousarray(np.asarray(self.seg_off, dtype=np.int32))
        self.seg_adapter = np.ascontiguousarray(np.asarray(self.seg_adapter, dtype=np.int32))
        self.scale = _f32(self.scale).reshape(-1)
        if self.rank is None:
            self.rank = np.array([a.shape[1] for a in self.A], dtype=np.int32)
        self.rank = np.ascontiguousarray(np.asarray(self.rank, dtype=np.int32))
        T, D = self.x.shape
        D2, K = self.W.shape
        assert D == D2, "x and W disagree on d"
        assert len(self.A) == len(self.B) == len(self.rank) == len(self.scale)
        for k, (a, b) in enumerate(zip(self.A, self.B)):
            r = int(self.rank[k])
            assert a.shape == (D, r), f"A[{k}] must be [d, r]"
            assert b.shape == (r, K), f"B[{k}] must be [r, k]"
        assert len(self.seg_off) == len(self.seg_adapter) + 1

    @property
    def T(self) -> int:
        return self.x.shape[0]

    @property
    def D(self) -> int:
        return self.x.shape[1]

    @property
    def K(self) -> int:
        return self.W.shape[1]

    @property
    def n_seg(self) -> int:
        return len(self.seg_adapter)

    @property
    def n_adapters(self) -> int:
        return len(self.A)

    def rows_of_adapter(self, k: int) -> np.ndarray:
        """Token rows of adapter k, in order."""
        parts = [np.arange(self.seg_off[s], self.seg_off[s + 1], dtype=np.int64)
                 for s in range(self.n_seg) if self.seg_adapter[s] == k]
        return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)

    def take_rows(self, rows) -> "Problem":
        """The same layer on a subset of the tokens: rows (sorted, unique) keep their segment,
        hence their adapter; segments that lose all their rows become empty.  Pure indexing -
        every token's outputs depend on its own row and its adapter only (section 2.4), so
        y, h, dx, g of the sub-problem are those rows of the full problem."""
        rows = np.asarray(rows, dtype=np.int64)
        assert rows.ndim == 1 and (len(rows) == 0 or (np.all(np.diff(rows) > 0) and rows[0] >= 0
                                                      and rows[-1] < self.T))
        off = np.searchsorted(rows, self.seg_off.astype(np.int64), side="left").astype(np.int32)
        return Problem(self.x[rows], self.W, self.A, self.B, off, self.seg_adapter, self.scale,
                       self.rank)
