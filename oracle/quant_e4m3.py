"""CPU oracle of the weight-only 8-bit expert weights -- TEST INFRASTRUCTURE ONLY.

The storage format is OCP "FP8 E4M3" (Micikevicius et al., "FP8 Formats for Deep Learning", 2022,
the variant without infinities): 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits;
exponent field 0 holds the subnormals m/8 * 2^-6; the code S.1111.111 is NaN; the largest finite
value is 1.75 * 2^8 = 448.  This is an extension on the MI355X side, not part of the paper; the
definitions below are written out from the format, in numpy fp64, and share nothing with the
library's kernels.  Only tests, the smoke check and the benchmark's baseline leg may import it.

    scale(W)    the smallest power of two s with max|W| <= 448 s (1 for an all-zero W)
    quantize    q = the e4m3 value nearest to W / s, ties to the even mantissa, as a byte
    dequantize  s * value(q)

The library hands its bytes out in a blocked order (16 rows x 64 columns per contiguous 1 KB, the
blocks of a 16-row group one after the other along the columns); ``blocked`` / ``unblocked``
restate that order with numpy reshapes so that tests can compare bytes element by element.
"""
from __future__ import annotations

import math

import numpy as np

E4M3_MAX = 448.0


def value_of_code(code: int) -> float:
    """The real number a byte stands for (NaN for 0x7f / 0xff)."""
    sign = -1.0 if code & 0x80 else 1.0
    ex = (code >> 3) & 0xF
    man = code & 0x7
    if ex == 0xF and man == 0x7:
        return float("nan")
    if ex == 0:
        return sign * (man / 8.0) * 2.0 ** -6
    return sign * (1.0 + man / 8.0) * 2.0 ** (ex - 7)


def code_values() -> np.ndarray:
    return np.array([value_of_code(c) for c in range(256)], dtype=np.float64)


def scale_of(absmax: float) -> float:
    if not absmax > 0.0:
        return 1.0
    n = math.ceil(math.log2(absmax / E4M3_MAX))
    # log2 of a ratio close to a power of two may land on either side: settle it exactly
    while absmax > E4M3_MAX * 2.0 ** n:
        n += 1
    while absmax <= E4M3_MAX * 2.0 ** (n - 1):
        n -= 1
    return 2.0 ** max(n, -126)


def nearest_code(v: np.ndarray) -> np.ndarray:
    """Element-wise nearest e4m3 value of |v| <= 448, ties to the even mantissa -> bytes.
    By search over the 127 non-negative finite codes (whose values ascend with the code)."""
    v = np.asarray(v, dtype=np.float64)
    grid = code_values()[:0x7F]                      # 0 .. 448, ascending
    a = np.abs(v)
    if a.size and a.max() > E4M3_MAX:
        raise ValueError("value beyond the e4m3 range")
    hi = np.searchsorted(grid, a, side="left")       # first code with value >= a
    hi = np.minimum(hi, 0x7E)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - grid[lo], grid[hi] - a
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))   # even code = even mantissa
    code = np.where(take_hi, hi, lo).astype(np.uint8)
    neg = np.signbit(v)
    return np.where(neg, code | 0x80, code).astype(np.uint8)


def quantize(w: np.ndarray):
    """w [E, ...] -> (q uint8 of the same shape, scale [E] float32), one scale per w[e]."""
    w = np.asarray(w, dtype=np.float64)
    E = w.shape[0]
    q = np.empty(w.shape, dtype=np.uint8)
    scale = np.empty(E, dtype=np.float32)
    for e in range(E):
        s = scale_of(float(np.abs(w[e]).max()) if w[e].size else 0.0)
        scale[e] = s
        q[e] = nearest_code(w[e] / s)
    return q, scale


def dequantize(q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """-> float64 array scale[e] * value(q[e])."""
    vals = code_values()[np.asarray(q, dtype=np.uint8)]
    shape = (len(scale),) + (1,) * (vals.ndim - 1)
    return vals * np.asarray(scale, dtype=np.float64).reshape(shape)


def blocked(q: np.ndarray) -> np.ndarray:
    """[E, rows, cols] bytes -> [E, rows * cols] in the library's order: element (n, k) at
    ((n // 16) * (cols // 64) + k // 64) * 1024 + (n % 16) * 64 + k % 64."""
    E, rows, cols = q.shape
    assert rows % 16 == 0 and cols % 64 == 0
    return q.reshape(E, rows // 16, 16, cols // 64, 64).transpose(0, 1, 3, 2, 4).reshape(E, rows * cols)


def unblocked(qb: np.ndarray, rows: int, cols: int) -> np.ndarray:
    """Inverse of ``blocked``: [E, rows * cols] -> [E, rows, cols]."""
    E = qb.shape[0]
    return qb.reshape(E, rows // 16, cols // 64, 16, 64).transpose(0, 1, 3, 2, 4).reshape(E, rows, cols)
