"""Seeded synthetic inputs shaped like the paper's packed-LoRA workloads.

This module only draws numbers and lays out segments; it contains none of the layer's
arithmetic, so that both the HIP library and the CPU oracle can be fed from it.

The paper fine-tunes Qwen-2.5 / Llama-3 models with 2-32 packed adapters of rank 8-128
(Table 1, Tables 7-8, section 5 setup) on text datasets that are not needed here: the layer is
dense linear algebra whose cost depends on shapes and token counts only.  The five
configurations below follow those shapes (Llama-3-8B / 70B projection sizes, seven LoRA-wrapped
projections per decoder layer as in appendix B); values are i.i.d. draws:

    x, dy ~ N(0, 1);  W ~ N(0, 1/d_in);  A ~ U(-1/sqrt(d_in), 1/sqrt(d_in));  B ~ N(0, var_B)

each rounded (nearest-even) to the I/O dtype before anyone sees it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 250802932


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array whose values are bf16-representable (round-nearest-even).

    Finite inputs only."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    w = u >> np.uint32(16)          # in-place steps below keep large inputs to one temporary
    w &= np.uint32(1)
    w += np.uint32(0x7FFF)
    w += u
    w &= np.uint32(0xFFFF0000)
    return w.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an array that already holds bf16-representable float32 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 values."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _round(a: np.ndarray, dtype: str) -> np.ndarray:
    return round_to_bf16(a) if dtype == "bf16" else np.ascontiguousarray(a, dtype=np.float32)


@dataclass
class Layout:
    """Segment packing of one batch: who owns which rows."""
    seg_off: np.ndarray       # [n_seg+1] int32
    seg_adapter: np.ndarray   # [n_seg] int32, -1 = base only
    rank: np.ndarray          # [n_adapters] int32
    scale: np.ndarray         # [n_adapters] float32

    @property
    def T(self) -> int:
        return int(self.seg_off[-1]) if len(self.seg_off) else 0

    @property
    def n_seg(self) -> int:
        return len(self.seg_adapter)

    @property
    def n_adapters(self) -> int:
        return len(self.rank)

    def sum_Lr(self) -> int:
        """Sum over segments of length x rank (size of the ragged low-rank activation)."""
        tot = 0
        for s in range(self.n_seg):
            k = int(self.seg_adapter[s])
            if k >= 0:
                tot += int(self.seg_off[s + 1] - self.seg_off[s]) * int(self.rank[k])
        return tot


@dataclass
class Tensors:
    x: np.ndarray
    W: np.ndarray
    A: List[np.ndarray]
    B: List[np.ndarray]
    dy: np.ndarray


@dataclass
class Linear:
    """One packed linear layer instance: shapes, dtype, layout, and how to draw its tensors."""
    name: str
    dtype: str                # "bf16" or "f32"
    D: int
    K: int
    layout: Layout
    var_B: float
    seed: int
    a_bound: Optional[float] = None   # None -> 1/sqrt(D)

    def flops_fwd_bwd(self) -> float:
        """4 T D K for the two base products plus 6 (D+K) sum(L r) for the low-rank ones."""
        T = self.layout.T
        return 4.0 * T * self.D * self.K + 6.0 * (self.D + self.K) * self.layout.sum_Lr()

    def tensors(self, want: Sequence[str] = ("x", "W", "A", "B", "dy")) -> Tensors:
        T, D, K = self.layout.T, self.D, self.K
        bound = self.a_bound if self.a_bound is not None else 1.0 / np.sqrt(D)

        def rng(tid):
            return np.random.default_rng(self.seed + tid)

        x = W = dy = None
        A: List[np.ndarray] = []
        B: List[np.ndarray] = []
        if "x" in want:
            x = _round(rng(1).standard_normal((T, D), dtype=np.float32), self.dtype)
        if "W" in want:
            W = rng(2).standard_normal((D, K), dtype=np.float32)
            W *= np.float32(1.0 / np.sqrt(D))
            W = _round(W, self.dtype)
        if "dy" in want:
            dy = _round(rng(3).standard_normal((T, K), dtype=np.float32), self.dtype)
        if "A" in want:
            for k, r in enumerate(self.layout.rank):
                a = rng(100 + k).uniform(-bound, bound, size=(D, int(r))).astype(np.float32)
                A.append(_round(a, self.dtype))
        if "B" in want:
            for k, r in enumerate(self.layout.rank):
                b = rng(500 + k).standard_normal((int(r), K), dtype=np.float32)
                b *= np.float32(np.sqrt(self.var_B))
                B.append(_round(b, self.dtype))
        return Tensors(x, W, A, B, dy)


def equal_layout(n_adapters: int, tokens_each: int, ranks: Sequence[int],
                 scales: Sequence[float]) -> Layout:
    off = np.arange(n_adapters + 1, dtype=np.int32) * np.int32(tokens_each)
    return Layout(off, np.arange(n_adapters, dtype=np.int32),
                  np.asarray(ranks, dtype=np.int32), np.asarray(scales, dtype=np.float32))


def unequal_lengths(rng: np.random.Generator, n: int, lo: int, hi: int, total: int) -> np.ndarray:
    """n integer lengths in [lo, hi] that sum to total, not aligned to anything."""
    assert n * lo <= total <= n * hi
    w = rng.uniform(0.0, 1.0, size=n)
    L = lo + np.floor((total - n * lo) * w / w.sum()).astype(np.int64)
    L = np.minimum(L, hi)
    i = 0
    while L.sum() < total:
        if L[i % n] < hi:
            L[i % n] += 1
        i += 1
    assert L.sum() == total and L.min() >= lo and L.max() <= hi
    return L


def _layout_from_lengths(L: np.ndarray, ranks: np.ndarray, scales: np.ndarray) -> Layout:
    off = np.zeros(len(L) + 1, dtype=np.int32)
    off[1:] = np.cumsum(L)
    return Layout(off, np.arange(len(L), dtype=np.int32), ranks.astype(np.int32),
                  scales.astype(np.float32))


def config(idx: int) -> List[Linear]:
    """The linears of benchmark configuration idx (1..5), in execution order."""
    seed = BASE_SEED + 1000 * idx
    if idx == 1:
        # tiny fp32 case: 2 adapters of rank 4 and 8, 128 tokens each, scale = 16 / r
        lay = equal_layout(2, 128, [4, 8], [16.0 / 4, 16.0 / 8])
        return [Linear("c1", "f32", 256, 256, lay, 0.01, seed, a_bound=1.0 / 16)]
    if idx == 2:
        # Llama-3-8B q_proj, 4 adapters x 2048 tokens, alpha = 2 r  ->  scale 2
        lay = equal_layout(4, 2048, [8, 16, 32, 64], [2.0] * 4)
        return [Linear("c2_q_proj", "bf16", 4096, 4096, lay, 0.02, seed)]
    if idx == 3:
        rng = np.random.default_rng(seed)
        ranks = rng.choice(np.array([8, 16, 32, 64, 128]), size=8)
        L = unequal_lengths(rng, 8, 512, 4096, 16384)
        lay = _layout_from_lengths(L, ranks, np.full(8, 2.0))
        return [Linear("c3_mlp_up", "bf16", 4096, 14336, lay, 0.02, seed + 10),
                Linear("c3_mlp_down", "bf16", 14336, 4096, lay, 0.02, seed + 20)]
    if idx == 4:
        ranks = np.array([16, 32] * 8)
        lay = equal_layout(16, 1024, ranks, [2.0] * 16)
        dims = [("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
                ("gate", 4096, 14336), ("up", 4096, 14336), ("down", 14336, 4096)]
        return [Linear(f"c4_{n}", "bf16", d, k, lay, 0.02, seed + 10 * (i + 1))
                for i, (n, d, k) in enumerate(dims)]
    if idx == 5:
        rng = np.random.default_rng(seed)
        raw = np.exp(rng.uniform(np.log(8.0), np.log(128.0), size=32))
        ranks = np.clip(8 * np.round(raw / 8.0), 8, 128).astype(np.int64)
        L = unequal_lengths(rng, 32, 256, 2048, 32768)
        lay = _layout_from_lengths(L, ranks, np.full(32, 2.0))
        return [Linear("c5_attn", "bf16", 8192, 8192, lay, 0.02, seed + 10),
                Linear("c5_mlp_up", "bf16", 8192, 28672, lay, 0.02, seed + 20)]
    raise ValueError("configuration index must be 1..5")


def small(name: str, dtype: str, D: int, K: int, lengths: Sequence[int],
          seg_adapter: Sequence[int], ranks: Sequence[int], scales: Sequence[float],
          seed: int = 7, var_B: float = 0.02) -> Linear:
    """Free-form small case for tests: any lengths (zero allowed), repeated or -1 adapters."""
    off = np.zeros(len(lengths) + 1, dtype=np.int32)
    off[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    lay = Layout(off, np.asarray(seg_adapter, dtype=np.int32), np.asarray(ranks, dtype=np.int32),
                 np.asarray(scales, dtype=np.float32))
    return Linear(name, dtype, D, K, lay, var_B, BASE_SEED + 77000 + seed)


def nf4_storage(n_elems: int, d_in: int, seed: int):
    """Synthetic 4-bit storage of a base weight with n_elems elements (a multiple of 64): uniformly random indices, two
    per byte, and per-block constants around 1.8 / sqrt(d_in), which gives the stored values about the variance
    1 / d_in of the dense synthetic weights (the 16 levels have a mean square of 0.30).  Returns (codes uint8
    [n_elems / 2], absmax fp32 [n_elems / 64]); nothing here knows the levels."""
    assert n_elems % 64 == 0
    rng = np.random.default_rng(BASE_SEED + 7919 * seed + 13)
    codes = rng.integers(0, 256, size=n_elems // 2, dtype=np.uint8)
    absmax = ((0.5 + rng.random(n_elems // 64)) * (1.8 / np.sqrt(d_in))).astype(np.float32)
    return codes, absmax
