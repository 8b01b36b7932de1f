"""Runs the HIP library on a workload and brings the results back as numpy arrays.

Only marshalling: torch owns the device memory, every step of the layer runs in libplora.
Outputs are pre-filled with NaN so that an element the kernels fail to write shows up, and every
output and the workspace sit between two 4 KB guard bands of a byte pattern that ``check_guards``
expects to find untouched (a write before the start or past the end of a buffer lands there).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from paper_2508_02932_amd import plora
from paper_2508_02932_amd import workloads as wl


def desc_of(lin: wl.Linear, w_layout: int = 0) -> plora.Desc:
    lay = lin.layout
    return plora.Desc(lay.T, lin.D, lin.K, lay.seg_off, lay.seg_adapter, lay.rank, lay.scale,
                      plora.PLORA_BF16 if lin.dtype == "bf16" else plora.PLORA_F32, w_layout)


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


GUARD_BYTES = 4096
GUARD_BYTE = 0xC5


def guarded(shape, dtype: torch.dtype, fill, guards: list, name: str) -> torch.Tensor:
    """A tensor of the given shape whose storage lies between two guard bands; registers the bands."""
    numel = int(np.prod(shape)) if len(shape) else 1
    nbytes = numel * torch.empty(0, dtype=dtype).element_size()
    pad = (-nbytes) % 256
    base = torch.full((GUARD_BYTES + nbytes + pad + GUARD_BYTES,), GUARD_BYTE, dtype=torch.uint8, device="cuda")
    view = base[GUARD_BYTES:GUARD_BYTES + nbytes].view(dtype).view(*shape)
    if fill is not None:
        view.fill_(fill)
    guards.append((name, base, nbytes))
    return view


def check_guards(p: "DeviceProblem") -> None:
    """Raises if any byte of a guard band changed (call after synchronising)."""
    for name, base, nbytes in p.guards:
        lo = base[:GUARD_BYTES]
        hi = base[GUARD_BYTES + nbytes:]
        assert bool((lo == GUARD_BYTE).all()), f"write before the start of {name}"
        assert bool((hi == GUARD_BYTE).all()), f"write past the end of {name}"


@dataclass
class DeviceProblem:
    lin: wl.Linear
    desc: plora.Desc
    x: torch.Tensor
    W: torch.Tensor
    A: List[torch.Tensor]
    B: List[torch.Tensor]
    dy: Optional[torch.Tensor]
    ws: torch.Tensor
    h: torch.Tensor
    y: torch.Tensor
    dx: torch.Tensor
    dA: List[torch.Tensor]
    dB: List[torch.Tensor]
    guards: list


def upload(lin: wl.Linear, t: wl.Tensors, w_layout: int = 0, lora_only: bool = False) -> DeviceProblem:
    """w_layout = plora.PLORA_W_OUT_IN hands the library W stored [d_out][d_in] (the same matrix, transposed in memory);
    lora_only sizes the workspace for the stand-alone low-rank calls."""
    d = desc_of(lin, w_layout)
    tdt = torch.bfloat16 if lin.dtype == "bf16" else torch.float32
    ws_bytes = plora.plora_lora_workspace_bytes(d) if lora_only else plora.plora_workspace_bytes(d)
    assert ws_bytes > 0
    nan = float("nan")
    T, D, K = lin.layout.T, lin.D, lin.K
    g: list = []
    return DeviceProblem(
        lin, d, to_dev(t.x, lin.dtype), to_dev(t.W.T if w_layout else t.W, lin.dtype),
        [to_dev(a, lin.dtype) for a in t.A], [to_dev(b, lin.dtype) for b in t.B],
        None if t.dy is None else to_dev(t.dy, lin.dtype),
        guarded((ws_bytes,), torch.uint8, None, g, "workspace"),
        guarded((max(plora.plora_h_elems(d), 1),), torch.float32, nan, g, "h_saved"),
        guarded((T, K), tdt, nan, g, "y"),
        guarded((T, D), tdt, nan, g, "dx"),
        [guarded((D, int(r)), torch.float32, nan, g, f"dA[{k}]") for k, r in enumerate(lin.layout.rank)],
        [guarded((int(r), K), torch.float32, nan, g, f"dB[{k}]") for k, r in enumerate(lin.layout.rank)],
        g)


def forward(p: DeviceProblem, save_h: bool = True):
    plora.plora_linear_fwd(p.desc, p.x, p.W, p.A, p.B, p.y, p.h if save_h else None, p.ws)


def backward(p: DeviceProblem, use_saved_h: bool = True, want_dx: bool = True, want_w: bool = True):
    plora.plora_linear_bwd(p.desc, p.x, p.W, p.A, p.B, p.dy, p.h if use_saved_h else None,
                           p.dx if want_dx else None, p.dA if want_w else None,
                           p.dB if want_w else None, p.ws)


def ragged_h_to_rows(lin: wl.Linear, h_flat: np.ndarray) -> np.ndarray:
    """Ragged saved activation -> [T, r_max] with zeros beyond each row's rank (the oracle's layout)."""
    lay = lin.layout
    pitch = int(lay.rank.max()) if lay.n_adapters else 1
    out = np.zeros((lay.T, pitch), dtype=np.float64)
    off = 0
    for s in range(lay.n_seg):
        k = int(lay.seg_adapter[s])
        lo, hi = int(lay.seg_off[s]), int(lay.seg_off[s + 1])
        if k < 0:
            continue
        r = int(lay.rank[k])
        out[lo:hi, :r] = h_flat[off:off + (hi - lo) * r].reshape(hi - lo, r)
        off += (hi - lo) * r
    return out


def lora_forward(p: DeviceProblem, save_h: bool = True):
    """Stand-alone low-rank forward: p.y must hold the base product on entry."""
    plora.plora_lora_fwd(p.desc, p.x, p.A, p.B, p.y, p.h if save_h else None, p.ws)


def lora_backward(p: DeviceProblem, use_saved_h: bool = True, want_dx: bool = True, want_w: bool = True):
    """Stand-alone low-rank backward: p.dx must hold dy W^T on entry."""
    plora.plora_lora_bwd(p.desc, p.x, p.A, p.B, p.dy, p.h if use_saved_h else None, p.dx if want_dx else None,
                         p.dA if want_w else None, p.dB if want_w else None, p.ws)
