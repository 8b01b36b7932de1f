"""4-bit NormalFloat (NF4) storage of a frozen base weight.  Test infrastructure only.

The paper runs packed LoRA on top of QLoRA (section 4 on LoRA variants; appendix on the A10
evaluation): the base weights are quantised to 4 bits, the LoRA computation is unchanged.  It does
not restate the storage format; this is NF4 as published with QLoRA (Dettmers et al., "QLoRA:
Efficient Finetuning of Quantized LLMs", section 3 and appendix E):

* the weight, flattened in memory order, is cut into blocks of 64 consecutive elements;
* each block keeps one fp32 constant, the largest magnitude in the block ("absmax");
* each element keeps a 4-bit index into a table of 16 values in [-1, 1] whose entries are quantiles
  of a standard normal, built so that 0 is represented exactly (8 positive levels from 9 evenly
  spaced probabilities between 0.9677083 and 0.5, 7 negative levels from 8 such probabilities, zero,
  all divided by the largest);
* an element's value is table[index] * absmax of its block.

Choices the publication leaves to the implementation, fixed here: two indices per byte, the element
with the even position in the high four bits; no second quantisation of the absmax constants; the
product is formed in fp32 (one correctly rounded multiplication, as fp32 hardware gives) and then
rounded to bf16, nearest even, when the layer runs in bf16.

The table is the 16 fp32 constants of the format as every stored NF4 weight assumes them.
``table_from_quantiles`` is the construction written out; the constants agree with it to 1.1e-7 (they
were first computed in fp32), which the pin tests check.
"""
from __future__ import annotations

import numpy as np

BLOCK = 64

TABLE = np.array([
    -1.0, -0.6961928009986877, -0.5250730514526367, -0.39491748809814453,
    -0.28444138169288635, -0.18477343022823334, -0.09105003625154495, 0.0,
    0.07958029955625534, 0.16093020141124725, 0.24611230194568634, 0.33791524171829224,
    0.44070982933044434, 0.5626170039176941, 0.7229568362236023, 1.0], dtype=np.float32)


def table_from_quantiles() -> np.ndarray:
    """The 16 levels from the quantile construction, fp64."""
    from scipy.stats import norm
    offset = 0.9677083
    positive = norm.ppf(np.linspace(offset, 0.5, 9)[:-1])        # 8 levels
    negative = -norm.ppf(np.linspace(offset, 0.5, 8)[:-1])       # 7 levels
    v = np.sort(np.concatenate([negative, [0.0], positive]))
    return v / v.max()


def _round_bf16(a32: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 (ties to even), returned as fp32."""
    u = a32.astype(np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def unpack(codes: np.ndarray, n: int) -> np.ndarray:
    """Bytes -> n four-bit indices: element 2i is the high half of byte i, element 2i+1 the low half."""
    codes = np.asarray(codes, dtype=np.uint8).ravel()
    assert n % 2 == 0 and codes.size == n // 2
    idx = np.empty(n, dtype=np.uint8)
    idx[0::2] = codes >> 4
    idx[1::2] = codes & 15
    return idx


def dequantize(codes: np.ndarray, absmax: np.ndarray, n: int, dtype: str) -> np.ndarray:
    """The n values of a stored weight, flat, as fp32 holding exactly what the layer computes with:
    fp32 products for dtype "f32", those rounded to bf16 for "bf16"."""
    assert n % BLOCK == 0
    absmax = np.asarray(absmax, dtype=np.float32).ravel()
    assert absmax.size == n // BLOCK
    level = TABLE[unpack(codes, n)]                                # fp32
    value = level * np.repeat(absmax, BLOCK)                       # fp32 * fp32 -> fp32, correctly rounded
    assert value.dtype == np.float32
    if dtype == "f32":
        return value
    assert dtype == "bf16"
    return _round_bf16(value)


def quantize(w: np.ndarray):
    """Nearest-level quantisation of a flat weight (n a multiple of 64): returns (codes, absmax).
    Used by tests to make stored weights from real ones; the layer itself only ever dequantises."""
    w = np.asarray(w, dtype=np.float64).ravel()
    n = w.size
    assert n % BLOCK == 0
    blocks = w.reshape(-1, BLOCK)
    absmax = np.abs(blocks).max(axis=1)
    safe = np.where(absmax > 0, absmax, 1.0)
    scaled = blocks / safe[:, None]
    idx = np.abs(scaled[:, :, None] - TABLE.astype(np.float64)[None, None, :]).argmin(axis=2).astype(np.uint8).ravel()
    codes = ((idx[0::2] << 4) | idx[1::2]).astype(np.uint8)
    return codes, absmax.astype(np.float32)
