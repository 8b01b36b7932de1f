"""ctypes binding of libplora (include/plora.h).  Argument marshalling only.

Every function here has the name and the meaning of the C entry point it calls; torch tensors
are used as owners of device memory and as the source of the HIP stream, nothing is computed in
Python.  The library must have been built (``python -m paper_2508_02932_amd.build`` or
``__graft_entry__.build()``); there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# PLORA_LIBRARY: another build of the same library (tuning runs of sweep_placement.py); normally unset
LIB_PATH = os.environ.get("PLORA_LIBRARY") or os.path.join(_HERE, "libplora.so")

PLORA_BF16, PLORA_F32 = 0, 1
PLORA_W_IN_OUT, PLORA_W_OUT_IN = 0, 1
PLORA_OK = 0
PLORA_MAX_RANK, PLORA_MAX_ADAPTERS, PLORA_MAX_SEGMENTS = 128, 256, 1024
KERNEL_CLASSES = {"gemm_fwd": 0, "gemm_dx": 1, "shrink": 2, "dh": 3, "db": 4, "da": 5, "prep": 6, "adamw": 7, "expand": 8, "nf4": 9}

EXPORTS = ["plora_status_string", "plora_validate", "plora_h_elems", "plora_workspace_bytes",
           "plora_build_metadata", "plora_linear_fwd", "plora_linear_fwd_noalloc", "plora_linear_bwd",
           "plora_set_kernel_timing", "plora_kernel_time", "plora_debug_metadata", "plora_adamw_step",
           "plora_lora_workspace_bytes", "plora_lora_fwd", "plora_lora_bwd",
           "plora_nf4_workspace_bytes", "plora_nf4_dequantize", "plora_linear_fwd_nf4", "plora_linear_bwd_nf4",
           "plora_group_workspace_bytes", "plora_group_fwd", "plora_group_bwd",
           "plora_plan_lora_bytes", "plora_plan_pack", "plora_plan_dtm", "plora_plan_schedule"]


class PloraError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"plora status {code}: {text}")
        self.code = code


class plora_desc(C.Structure):
    _fields_ = [("T", C.c_int64), ("d_in", C.c_int64), ("d_out", C.c_int64),
                ("n_seg", C.c_int32), ("n_adapters", C.c_int32),
                ("seg_off", C.c_void_p), ("seg_adapter", C.c_void_p),
                ("rank", C.c_void_p), ("scale", C.c_void_p), ("dtype", C.c_int32), ("w_layout", C.c_int32)]


class plora_group(C.Structure):
    _fields_ = [("n_proj", C.c_int32), ("desc", C.POINTER(plora_desc))]


class plora_plan_model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int64), ("kv_hidden", C.c_int64), ("inter", C.c_int64),
                ("c_prec", C.c_double), ("c_grad", C.c_double)]


class plora_plan_lora(C.Structure):
    _fields_ = [("rank", C.c_int32), ("batch", C.c_int32), ("seq", C.c_int32), ("targets", C.c_uint32)]


class plora_plan_sharding(C.Structure):
    _fields_ = [("zero_level", C.c_int32), ("d_tp", C.c_int32), ("d_pp", C.c_int32), ("d_fsdp", C.c_int32)]


class plora_plan_problem(C.Structure):
    _fields_ = [("n_configs", C.c_int32), ("n_degrees", C.c_int32), ("rank", C.c_void_p), ("mem", C.c_void_p),
                ("mem_base", C.c_double), ("mem_gpu", C.c_double), ("load", C.c_double),
                ("t_base", C.c_void_p), ("t_config", C.c_void_p)]


class plora_plan_job(C.Structure):
    _fields_ = [("first", C.c_int32), ("count", C.c_int32), ("gpus", C.c_int32), ("proved", C.c_int32),
                ("value", C.c_double), ("start", C.c_double), ("end", C.c_double)]


class plora_plan_summary(C.Structure):
    _fields_ = [("makespan", C.c_double), ("gpu_work", C.c_double), ("tail_bound", C.c_double),
                ("n_jobs", C.c_int32), ("n_unscheduled", C.c_int32), ("all_proved", C.c_int32)]


class plora_adamw_hparams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("step", C.c_int32), ("grad_scale", C.c_float)]


class plora_adamw_side(C.Structure):
    _fields_ = [("param", C.c_void_p), ("master", C.c_void_p), ("grad", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p)]


class plora_debug_info(C.Structure):
    _fields_ = ([("n_tiles", C.c_int64)]
                + [(n, C.c_int32) for n in ("n_seg", "n_adapters", "n_blocks", "max_r16", "seg_stride", "ad_stride",
                                            "tile_stride", "desc_words")]
                + [(n, C.c_uint64) for n in ("off_hdr", "off_seg", "off_ad", "off_tile", "off_blk_seg", "off_seg_list",
                                             "table_bytes")]
                + [(n, C.c_int32) for n in ("shrink_splits", "dh_splits", "da_splits", "da_tile_cols", "db_splits",
                                            "db_tile_cols", "r16_total", "n_active")]
                + [(n, C.c_uint64) for n in ("ws_zero", "ws_meta", "ws_desc", "ws_at", "ws_ap", "ws_hb", "ws_zt_h",
                                             "ws_zt_g", "ws_hf", "ws_gf", "ws_part", "ws_wpart", "ws_total", "h_elems",
                                             "off_tile_order")])


# numpy views of the records of the table image (include/plora_debug.h)
SEG_DTYPE = np.dtype([(n, "<i4") for n in ("row0", "row1", "adapter", "r", "rp", "r16", "blk0", "lp")]
                     + [(n, "<i8") for n in ("h_off", "hb_off", "zt_off")])
AD_DTYPE = np.dtype([(n, "<u8") for n in ("A", "B", "dA", "dB")] + [("r", "<i4"), ("rp", "<i4"), ("r16", "<i4"),
                    ("scale", "<f4"), ("at_off", "<i8"), ("ap_off", "<i8")]
                    + [(n, "<i4") for n in ("r16_off", "by_tokens", "seg_list0", "n_own", "tokens", "reserved")]
                    + [("ext_b", "<u8")])
_GSEG = [("row0", "<i4"), ("row1", "<i4"), ("rp", "<i4"), ("r", "<i4"), ("hb_off", "<i8"), ("B", "<u8"), ("ap_off", "<i8")]
TILE_DTYPE = np.dtype([(n, "<i4") for n in ("n_ext", "n_own", "first_seg", "third_seg")]
                      + [("s", np.dtype(_GSEG), (2,))])
HDR_DTYPE = np.dtype([("T", "<i8"), ("D", "<i8"), ("K", "<i8")] + [(n, "<i4") for n in ("n_seg", "n_adapters", "n_blocks", "max_r16", "w_out_in", "reserved")]
                     + [("at_base", "<u8")])

_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2508_02932_amd.build)")
        L = C.CDLL(LIB_PATH)
        L.plora_status_string.restype = C.c_char_p
        L.plora_status_string.argtypes = [C.c_int]
        L.plora_validate.restype = C.c_int
        L.plora_validate.argtypes = [C.POINTER(plora_desc)]
        L.plora_h_elems.restype = C.c_size_t
        L.plora_h_elems.argtypes = [C.POINTER(plora_desc)]
        L.plora_workspace_bytes.restype = C.c_size_t
        L.plora_workspace_bytes.argtypes = [C.POINTER(plora_desc)]
        L.plora_build_metadata.restype = C.c_int64
        L.plora_build_metadata.argtypes = [C.POINTER(plora_desc), C.c_int32, C.c_void_p, C.c_void_p, C.c_int64]
        L.plora_linear_fwd.restype = C.c_int
        L.plora_linear_fwd.argtypes = [C.POINTER(plora_desc)] + [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p]
        L.plora_linear_fwd_noalloc.restype = C.c_int
        L.plora_linear_fwd_noalloc.argtypes = [C.POINTER(plora_desc)] + [C.c_void_p] * 7
        L.plora_linear_bwd.restype = C.c_int
        L.plora_linear_bwd.argtypes = [C.POINTER(plora_desc)] + [C.c_void_p] * 10 + [C.c_size_t, C.c_void_p]
        L.plora_lora_workspace_bytes.restype = C.c_size_t
        L.plora_lora_workspace_bytes.argtypes = [C.POINTER(plora_desc)]
        L.plora_lora_fwd.restype = C.c_int
        L.plora_lora_fwd.argtypes = [C.POINTER(plora_desc)] + [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        L.plora_lora_bwd.restype = C.c_int
        L.plora_lora_bwd.argtypes = [C.POINTER(plora_desc)] + [C.c_void_p] * 9 + [C.c_size_t, C.c_void_p]
        L.plora_nf4_workspace_bytes.restype = C.c_size_t
        L.plora_nf4_workspace_bytes.argtypes = [C.POINTER(plora_desc)]
        L.plora_nf4_dequantize.restype = C.c_int
        L.plora_nf4_dequantize.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
        L.plora_linear_fwd_nf4.restype = C.c_int
        L.plora_linear_fwd_nf4.argtypes = [C.POINTER(plora_desc)] + [C.c_void_p] * 8 + [C.c_size_t, C.c_void_p]
        L.plora_linear_bwd_nf4.restype = C.c_int
        L.plora_linear_bwd_nf4.argtypes = [C.POINTER(plora_desc)] + [C.c_void_p] * 11 + [C.c_size_t, C.c_void_p]
        L.plora_group_workspace_bytes.restype = C.c_size_t
        L.plora_group_workspace_bytes.argtypes = [C.POINTER(plora_group)]
        L.plora_group_fwd.restype = C.c_int
        L.plora_group_fwd.argtypes = [C.POINTER(plora_group)] + [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p]
        L.plora_group_bwd.restype = C.c_int
        L.plora_group_bwd.argtypes = [C.POINTER(plora_group)] + [C.c_void_p] * 11 + [C.c_size_t, C.c_void_p]
        L.plora_plan_lora_bytes.restype = C.c_double
        L.plora_plan_lora_bytes.argtypes = [C.POINTER(plora_plan_model), C.POINTER(plora_plan_lora), C.POINTER(plora_plan_sharding)]
        L.plora_plan_pack.restype = C.c_int
        L.plora_plan_pack.argtypes = [C.POINTER(plora_plan_problem), C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(plora_plan_job)]
        L.plora_plan_dtm.restype = C.c_int
        L.plora_plan_dtm.argtypes = [C.POINTER(plora_plan_problem), C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                     C.POINTER(C.c_int32), C.c_void_p]
        L.plora_plan_schedule.restype = C.c_int
        L.plora_plan_schedule.argtypes = [C.POINTER(plora_plan_problem), C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                          C.POINTER(plora_plan_summary)]
        L.plora_set_kernel_timing.restype = None
        L.plora_set_kernel_timing.argtypes = [C.c_int]
        L.plora_kernel_time.restype = C.c_int
        L.plora_kernel_time.argtypes = [C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_int)]
        L.plora_adamw_step.restype = C.c_int
        L.plora_adamw_step.argtypes = [C.POINTER(plora_desc), C.POINTER(plora_adamw_side), C.POINTER(plora_adamw_side),
                                       C.POINTER(plora_adamw_hparams), C.c_void_p]
        L.plora_debug_metadata.restype = C.c_int
        L.plora_debug_metadata.argtypes = [C.POINTER(plora_desc), C.POINTER(plora_debug_info), C.c_void_p, C.c_size_t]
        _lib = L
    return _lib


@dataclass
class Desc:
    """Host-side description of one call; keeps the numpy arrays the C struct points at alive."""
    T: int
    d_in: int
    d_out: int
    seg_off: np.ndarray
    seg_adapter: np.ndarray
    rank: np.ndarray
    scale: np.ndarray
    dtype: int
    w_layout: int = 0       # PLORA_W_IN_OUT; PLORA_W_OUT_IN: W is stored [d_out][d_in]

    def __post_init__(self):
        self.seg_off = np.ascontiguousarray(self.seg_off, dtype=np.int32)
        self.seg_adapter = np.ascontiguousarray(self.seg_adapter, dtype=np.int32)
        self.rank = np.ascontiguousarray(self.rank, dtype=np.int32)
        self.scale = np.ascontiguousarray(self.scale, dtype=np.float32)
        self.c = plora_desc(self.T, self.d_in, self.d_out, len(self.seg_adapter), len(self.rank),
                            self.seg_off.ctypes.data, self.seg_adapter.ctypes.data,
                            self.rank.ctypes.data if len(self.rank) else None,
                            self.scale.ctypes.data if len(self.scale) else None, self.dtype, self.w_layout)

    @property
    def ref(self):
        return C.byref(self.c)


def _check(code: int):
    if code != PLORA_OK:
        raise PloraError(code, plora_status_string(code))


def plora_status_string(code: int) -> str:
    return lib().plora_status_string(int(code)).decode()


def plora_validate(d: Desc) -> int:
    return int(lib().plora_validate(d.ref))


def plora_h_elems(d: Desc) -> int:
    return int(lib().plora_h_elems(d.ref))


def plora_workspace_bytes(d: Desc) -> int:
    return int(lib().plora_workspace_bytes(d.ref))


def plora_build_metadata(d: Desc, block_rows: int):
    """(h_off[n_seg+1] int64, blocks[n, 4] int32) or raises on an invalid description."""
    n = int(lib().plora_build_metadata(d.ref, block_rows, None, None, 0))
    if n < 0:
        raise PloraError(-1, "invalid description")
    h_off = np.zeros(len(d.seg_adapter) + 1, dtype=np.int64)
    blocks = np.zeros((max(n, 1), 4), dtype=np.int32)
    n2 = int(lib().plora_build_metadata(d.ref, block_rows, h_off.ctypes.data, blocks.ctypes.data, n))
    assert n2 == n
    return h_off, blocks[:n]


def parse_tables(info: plora_debug_info, image: np.ndarray) -> dict:
    """Splits a table image (uint8 array, as exported or as read back from the workspace) into its records."""
    assert info.seg_stride == SEG_DTYPE.itemsize and info.ad_stride == AD_DTYPE.itemsize
    assert info.tile_stride == TILE_DTYPE.itemsize
    buf = np.ascontiguousarray(image, dtype=np.uint8)

    def take(off, dtype, n):
        return np.frombuffer(buf, dtype=dtype, count=n, offset=int(off)).copy()

    tabs = {"hdr": take(info.off_hdr, HDR_DTYPE, 1)[0], "seg": take(info.off_seg, SEG_DTYPE, info.n_seg),
            "ad": take(info.off_ad, AD_DTYPE, info.n_adapters), "tile": take(info.off_tile, TILE_DTYPE, info.n_tiles),
            "blk_seg": take(info.off_blk_seg, "<i4", info.n_blocks)}
    n_list = int(tabs["ad"]["n_own"].sum()) if info.n_adapters else 0
    tabs["seg_list"] = take(info.off_seg_list, "<i4", n_list)
    tabs["tile_order"] = take(info.off_tile_order, "<i4", info.n_tiles)
    return tabs


def plora_debug_metadata(d: Desc):
    """(info, tables) - the metadata exactly as the kernels read it, built on the host (no device)."""
    info = plora_debug_info()
    if lib().plora_debug_metadata(d.ref, C.byref(info), None, 0) != 0:
        raise PloraError(-1, "invalid description")
    image = np.zeros(int(info.table_bytes), dtype=np.uint8)
    if lib().plora_debug_metadata(d.ref, C.byref(info), image.ctypes.data, image.nbytes) != 0:
        raise PloraError(-1, "plora_debug_metadata failed")
    return info, parse_tables(info, image), image


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _ptr_table(tensors: Optional[Sequence]):
    if tensors is None:
        return None, None
    arr = (C.c_void_p * max(len(tensors), 1))(*[int(t.data_ptr()) for t in tensors])
    return arr, C.cast(arr, C.c_void_p)


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) or None


def plora_linear_fwd(d: Desc, x, W, A: Sequence, B: Sequence, y, h_saved, workspace, stream=None) -> None:
    """Enqueues the forward call; tensors are torch device tensors (h_saved may be None)."""
    ka, pa = _ptr_table(A)
    kb, pb = _ptr_table(B)
    code = lib().plora_linear_fwd(d.ref, _ptr(x), _ptr(W), pa, pb, _ptr(y), _ptr(h_saved),
                                  _ptr(workspace), workspace.numel() * workspace.element_size(),
                                  _stream(stream))
    _check(code)


NOALLOC_SCRATCH_BYTES = 64 << 20


def plora_linear_fwd_noalloc(d: Desc, x, W, A: Sequence, B: Sequence, y, h_saved, stream=None) -> None:
    """Forward on the library's own per-GPU scratch array (no workspace argument, nothing allocated)."""
    ka, pa = _ptr_table(A)
    kb, pb = _ptr_table(B)
    code = lib().plora_linear_fwd_noalloc(d.ref, _ptr(x), _ptr(W), pa, pb, _ptr(y), _ptr(h_saved), _stream(stream))
    _check(code)


def plora_linear_bwd(d: Desc, x, W, A: Sequence, B: Sequence, dy, h_saved, dx, dA: Optional[Sequence],
                     dB: Optional[Sequence], workspace, stream=None) -> None:
    """Enqueues the backward call; dx may be None, dA and dB may both be None."""
    ka, pa = _ptr_table(A)
    kb, pb = _ptr_table(B)
    kda, pda = _ptr_table(dA)
    kdb, pdb = _ptr_table(dB)
    code = lib().plora_linear_bwd(d.ref, _ptr(x), _ptr(W), pa, pb, _ptr(dy), _ptr(h_saved), _ptr(dx),
                                  pda, pdb, _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream))
    _check(code)


def plora_lora_workspace_bytes(d: Desc) -> int:
    return int(lib().plora_lora_workspace_bytes(d.ref))


def plora_lora_fwd(d: Desc, x, A: Sequence, B: Sequence, y, h_saved, workspace, stream=None) -> None:
    """Enqueues the stand-alone low-rank forward: y (holding the base product) += scale_k (x A_k) B_k."""
    ka, pa = _ptr_table(A)
    kb, pb = _ptr_table(B)
    _check(lib().plora_lora_fwd(d.ref, _ptr(x), pa, pb, _ptr(y), _ptr(h_saved), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)))


def plora_lora_bwd(d: Desc, x, A: Sequence, B: Sequence, dy, h_saved, dx, dA: Optional[Sequence],
                   dB: Optional[Sequence], workspace, stream=None) -> None:
    """Enqueues the stand-alone low-rank backward: dA, dB, and dx (holding dy W^T, may be None) += g A_k^T."""
    ka, pa = _ptr_table(A)
    kb, pb = _ptr_table(B)
    kda, pda = _ptr_table(dA)
    kdb, pdb = _ptr_table(dB)
    _check(lib().plora_lora_bwd(d.ref, _ptr(x), pa, pb, _ptr(dy), _ptr(h_saved), _ptr(dx), pda, pdb, _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)))


class Group:
    """Projections that read the same x; keeps the array of C descriptions (and the Desc objects behind it) alive."""

    def __init__(self, descs: Sequence[Desc]):
        self.descs = list(descs)
        self.arr = (plora_desc * max(len(self.descs), 1))(*[d.c for d in self.descs])
        self.c = plora_group(len(self.descs), self.arr)

    @property
    def ref(self):
        return C.byref(self.c)


def _ptr_array(tensors: Optional[Sequence]):
    """HOST array of device pointers (entries may be None)."""
    if tensors is None:
        return None, None
    arr = (C.c_void_p * max(len(tensors), 1))(*[None if t is None else int(t.data_ptr()) for t in tensors])
    return arr, C.cast(arr, C.c_void_p)


def _table_array(tables: Optional[Sequence]):
    """HOST array of HOST pointer tables (entries may be None)."""
    if tables is None:
        return None, None
    keep = [_ptr_table(t) for t in tables]
    arr = (C.c_void_p * max(len(tables), 1))(*[None if k[1] is None else k[1].value for k in keep])
    return (keep, arr), C.cast(arr, C.c_void_p)


def plora_group_workspace_bytes(g: Group) -> int:
    return int(lib().plora_group_workspace_bytes(g.ref))


def plora_group_fwd(g: Group, x, W: Sequence, A: Sequence[Sequence], B: Sequence[Sequence], y: Sequence,
                    h_saved: Optional[Sequence], workspace, stream=None) -> None:
    """Enqueues the forward of every projection of the group on one x (entry p of each list belongs to projection p)."""
    kw, pw = _ptr_array(W)
    ka, pa = _table_array(A)
    kb, pb = _table_array(B)
    ky, py = _ptr_array(y)
    kh, ph = _ptr_array(h_saved)
    _check(lib().plora_group_fwd(g.ref, _ptr(x), pw, pa, pb, py, ph, _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream)))


def plora_group_bwd(g: Group, x, W: Sequence, A: Sequence[Sequence], B: Sequence[Sequence], dy: Sequence,
                    h_saved: Optional[Sequence], dx: Optional[Sequence], dA: Optional[Sequence], dB: Optional[Sequence],
                    workspace, stream=None, dx_sum=None) -> None:
    """Enqueues the backward of every projection of the group.  dx[p] is projection p's own input gradient; dx_sum
    (instead of dx) receives their sum, the gradient of the shared input."""
    kw, pw = _ptr_array(W)
    ka, pa = _table_array(A)
    kb, pb = _table_array(B)
    kdy, pdy = _ptr_array(dy)
    kh, ph = _ptr_array(h_saved)
    kdx, pdx = _ptr_array(dx)
    kda, pda = _table_array(dA)
    kdb, pdb = _table_array(dB)
    _check(lib().plora_group_bwd(g.ref, _ptr(x), pw, pa, pb, pdy, ph, pdx, _ptr(dx_sum), pda, pdb, _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream)))


# ---- packing planner (host only) --------------------------------------------------------------------------

class PlanProblem:
    """Host-side planner input; keeps the numpy arrays the C struct points at alive.  t_config is [n_degrees][n]."""

    def __init__(self, rank, mem, mem_base: float, mem_gpu: float, load: float, t_base, t_config):
        self.rank = np.ascontiguousarray(rank, dtype=np.int32)
        self.mem = np.ascontiguousarray(mem, dtype=np.float64)
        self.t_base = np.ascontiguousarray(t_base, dtype=np.float64)
        self.t_config = np.ascontiguousarray(t_config, dtype=np.float64).reshape(len(self.t_base), len(self.rank))
        self.c = plora_plan_problem(len(self.rank), len(self.t_base), self.rank.ctypes.data, self.mem.ctypes.data,
                                    mem_base, mem_gpu, load, self.t_base.ctypes.data, self.t_config.ctypes.data)

    @property
    def ref(self):
        return C.byref(self.c)


def _jobs_to_py(jobs, n_jobs: int, cfg: np.ndarray):
    return [{"configs": cfg[j.first:j.first + j.count].tolist(), "gpus": int(j.gpus), "value": float(j.value),
             "proved": bool(j.proved), "start": float(j.start), "end": float(j.end)} for j in jobs[:n_jobs]]


def _avail(p: PlanProblem, avail):
    if avail is None:
        return None, None
    a = np.zeros(len(p.rank), dtype=np.uint8)
    a[list(avail)] = 1
    return a, a.ctypes.data


def plora_plan_lora_bytes(model: dict, cfg: dict, sharding: Optional[dict] = None) -> float:
    m = plora_plan_model(**model)
    c = plora_plan_lora(**cfg)
    s = plora_plan_sharding(**sharding) if sharding else None
    return float(lib().plora_plan_lora_bytes(C.byref(m), C.byref(c), C.byref(s) if s else None))


def plora_plan_pack(p: PlanProblem, degree_index: int, avail=None) -> dict:
    """F(D, K) on the configurations listed in avail (None: all)."""
    cfg = np.zeros(len(p.rank), dtype=np.int32)
    job = plora_plan_job()
    keep, ap = _avail(p, avail)
    _check(lib().plora_plan_pack(p.ref, degree_index, ap, cfg.ctypes.data, C.byref(job)))
    return _jobs_to_py([job], 1, cfg)[0]


def plora_plan_dtm(p: PlanProblem, gpus: int, avail=None) -> list:
    cfg = np.zeros(len(p.rank), dtype=np.int32)
    jobs = (plora_plan_job * max(gpus, 1))()
    n = C.c_int32(0)
    keep, ap = _avail(p, avail)
    _check(lib().plora_plan_dtm(p.ref, gpus, ap, C.cast(jobs, C.c_void_p), max(gpus, 1), C.byref(n), cfg.ctypes.data))
    return _jobs_to_py(jobs, n.value, cfg)


def plora_plan_schedule(p: PlanProblem, gpus: int) -> dict:
    n = len(p.rank)
    cfg = np.zeros(n, dtype=np.int32)
    jobs = (plora_plan_job * n)()
    s = plora_plan_summary()
    _check(lib().plora_plan_schedule(p.ref, gpus, C.cast(jobs, C.c_void_p), n, cfg.ctypes.data, C.byref(s)))
    return {"jobs": _jobs_to_py(jobs, s.n_jobs, cfg), "makespan": float(s.makespan), "gpu_work": float(s.gpu_work),
            "tail_bound": float(s.tail_bound), "unscheduled": cfg[n - s.n_unscheduled:].tolist() if s.n_unscheduled else [],
            "all_proved": bool(s.all_proved)}


def plora_nf4_workspace_bytes(d: Desc) -> int:
    return int(lib().plora_nf4_workspace_bytes(d.ref))


def plora_nf4_dequantize(codes, absmax, n_elems: int, dtype: int, out, stream=None) -> None:
    """Enqueues the expansion of an NF4 weight: out[i] = level[index_i] * absmax[i // 64]."""
    _check(lib().plora_nf4_dequantize(_ptr(codes), _ptr(absmax), int(n_elems), int(dtype), _ptr(out), _stream(stream)))


def plora_linear_fwd_nf4(d: Desc, x, W_codes, W_absmax, A: Sequence, B: Sequence, y, h_saved, workspace, stream=None) -> None:
    """plora_linear_fwd on an NF4 base weight (expanded into the workspace first)."""
    ka, pa = _ptr_table(A)
    kb, pb = _ptr_table(B)
    _check(lib().plora_linear_fwd_nf4(d.ref, _ptr(x), _ptr(W_codes), _ptr(W_absmax), pa, pb, _ptr(y), _ptr(h_saved),
                                      _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def plora_linear_bwd_nf4(d: Desc, x, W_codes, W_absmax, A: Sequence, B: Sequence, dy, h_saved, dx,
                         dA: Optional[Sequence], dB: Optional[Sequence], workspace, stream=None) -> None:
    """plora_linear_bwd on an NF4 base weight."""
    ka, pa = _ptr_table(A)
    kb, pb = _ptr_table(B)
    kda, pda = _ptr_table(dA)
    kdb, pdb = _ptr_table(dB)
    _check(lib().plora_linear_bwd_nf4(d.ref, _ptr(x), _ptr(W_codes), _ptr(W_absmax), pa, pb, _ptr(dy), _ptr(h_saved),
                                      _ptr(dx), pda, pdb, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)))


def plora_adamw_step(d: Desc, A_side: dict, B_side: dict, hparams: Sequence, stream=None) -> None:
    """Enqueues the per-adapter AdamW step.  A_side / B_side: dicts with the keys param, master, grad, m, v, each a
    list of n_adapters device tensors (param or master may be None); hparams: one (lr, beta1, beta2, eps,
    weight_decay, step[, grad_scale]) tuple per adapter (grad_scale: the adapter's multiplier on its gradient, 1 if left out)."""
    keep = []

    def side(s):
        tabs = []
        for key in ("param", "master", "grad", "m", "v"):
            arr, ptr = _ptr_table(s.get(key))
            keep.append(arr)
            tabs.append(ptr)
        return plora_adamw_side(*tabs)

    sa, sb = side(A_side), side(B_side)
    hp = (plora_adamw_hparams * max(len(hparams), 1))(*[plora_adamw_hparams(*(tuple(h) + (1.0,))[:7]) for h in hparams])
    _check(lib().plora_adamw_step(d.ref, C.byref(sa), C.byref(sb), hp, _stream(stream)))


def plora_set_kernel_timing(enabled: bool) -> None:
    lib().plora_set_kernel_timing(1 if enabled else 0)


def plora_kernel_time(kernel_class):
    """(total milliseconds, number of brackets) recorded for one kernel class since timing was enabled."""
    if isinstance(kernel_class, str):
        kernel_class = KERNEL_CLASSES[kernel_class]
    ms, n = C.c_float(0), C.c_int(0)
    if lib().plora_kernel_time(int(kernel_class), C.byref(ms), C.byref(n)) != 0:
        raise PloraError(-1, "plora_kernel_time failed")
    return float(ms.value), int(n.value)
