"""ctypes front end of the plain-C scalar-loop oracle (``plora_oracle.c``).

Test infrastructure only.  ``build()`` compiles the C file with gcc; the functions below only
marshal numpy arrays, the arithmetic is all in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Tuple

import numpy as np

from .problem import Problem

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "plora_oracle.c")
_LIB = os.path.join(_HERE, "libplora_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle (plain gcc, OpenMP over independent outputs, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-mavx2", "-ffp-contract=off", "-fopenmp",
               "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class _CProblem(C.Structure):
    _fields_ = [("T", C.c_int64), ("D", C.c_int64), ("K", C.c_int64),
                ("n_seg", C.c_int32), ("n_adapters", C.c_int32),
                ("seg_off", C.c_void_p), ("seg_adapter", C.c_void_p),
                ("rank", C.c_void_p), ("scale", C.c_void_p),
                ("x", C.c_void_p), ("W", C.c_void_p),
                ("A", C.c_void_p), ("B", C.c_void_p)]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.plora_oracle_threads.restype = C.c_int
        for name in ("plora_oracle_check", "plora_oracle_fwd_rows", "plora_oracle_bwd_rows",
                     "plora_oracle_grad_adapter"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def threads() -> int:
    """Threads the C oracle will use (OpenMP's maximum for this process)."""
    return int(_load().plora_oracle_threads())


def _marshal(p: Problem):
    """Returns (struct, keepalive list)."""
    n = p.n_adapters
    PtrArr = C.c_void_p * max(n, 1)
    a_ptrs = PtrArr(*[a.ctypes.data for a in p.A]) if n else PtrArr()
    b_ptrs = PtrArr(*[b.ctypes.data for b in p.B]) if n else PtrArr()
    s = _CProblem(p.T, p.D, p.K, p.n_seg, n,
                  p.seg_off.ctypes.data, p.seg_adapter.ctypes.data,
                  p.rank.ctypes.data, p.scale.ctypes.data,
                  p.x.ctypes.data, p.W.ctypes.data,
                  C.cast(a_ptrs, C.c_void_p), C.cast(b_ptrs, C.c_void_p))
    return s, (a_ptrs, b_ptrs, p)


def _check_rc(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def check(p: Problem) -> int:
    s, keep = _marshal(p)
    return int(_load().plora_oracle_check(C.byref(s)))


def _rows(p: Problem, rows) -> np.ndarray:
    if rows is None:
        return np.arange(p.T, dtype=np.int64)
    return np.ascontiguousarray(np.asarray(rows, dtype=np.int64))


def fwd_rows(p: Problem, rows=None) -> Tuple[np.ndarray, np.ndarray]:
    """(y[len(rows), K], h[len(rows), r_max]) for the listed tokens (all tokens if None).

    h is zero beyond the rank of the token's adapter (and all zero for adapter -1)."""
    rows = _rows(p, rows)
    pitch = int(p.rank.max()) if p.n_adapters else 1
    y = np.empty((len(rows), p.K), dtype=np.float64)
    h = np.empty((len(rows), pitch), dtype=np.float64)
    s, keep = _marshal(p)
    rc = _load().plora_oracle_fwd_rows(C.byref(s), C.c_int64(len(rows)),
                                       C.c_void_p(rows.ctypes.data), C.c_int32(pitch),
                                       C.c_void_p(h.ctypes.data), C.c_void_p(y.ctypes.data))
    _check_rc(rc, "fwd_rows")
    return y, h


def bwd_rows(p: Problem, dy: np.ndarray, rows=None) -> Tuple[np.ndarray, np.ndarray]:
    """(dx[len(rows), D], g[len(rows), r_max]) for the listed tokens (all tokens if None)."""
    rows = _rows(p, rows)
    dy = np.ascontiguousarray(np.asarray(dy, dtype=np.float32))
    assert dy.shape == (p.T, p.K)
    pitch = int(p.rank.max()) if p.n_adapters else 1
    dx = np.empty((len(rows), p.D), dtype=np.float64)
    g = np.empty((len(rows), pitch), dtype=np.float64)
    s, keep = _marshal(p)
    rc = _load().plora_oracle_bwd_rows(C.byref(s), C.c_void_p(dy.ctypes.data),
                                       C.c_int64(len(rows)), C.c_void_p(rows.ctypes.data),
                                       C.c_int32(pitch), C.c_void_p(g.ctypes.data),
                                       C.c_void_p(dx.ctypes.data))
    _check_rc(rc, "bwd_rows")
    return dx, g


def grad_adapter(p: Problem, dy: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """(dA_k[D, r_k], dB_k[r_k, K]) summed over every token of adapter k."""
    dy = np.ascontiguousarray(np.asarray(dy, dtype=np.float32))
    assert dy.shape == (p.T, p.K)
    r = int(p.rank[k])
    dA = np.empty((p.D, r), dtype=np.float64)
    dB = np.empty((r, p.K), dtype=np.float64)
    s, keep = _marshal(p)
    rc = _load().plora_oracle_grad_adapter(C.byref(s), C.c_void_p(dy.ctypes.data), C.c_int32(k),
                                           C.c_void_p(dA.ctypes.data), C.c_void_p(dB.ctypes.data))
    _check_rc(rc, "grad_adapter")
    return dA, dB


def forward(p: Problem) -> Tuple[np.ndarray, np.ndarray]:
    """All rows: (y[T, K], h[T, r_max])."""
    return fwd_rows(p, None)


def backward(p: Problem, dy: np.ndarray
             ) -> Tuple[np.ndarray, np.ndarray, List[np.ndarray], List[np.ndarray]]:
    """All rows and all adapters: (dx, g, [dA_k], [dB_k])."""
    dx, g = bwd_rows(p, dy, None)
    dA, dB = [], []
    for k in range(p.n_adapters):
        a, b = grad_adapter(p, dy, k)
        dA.append(a)
        dB.append(b)
    return dx, g, dA, dB
