"""CPU oracle of the weight-only 4-bit expert weights with block scales -- TEST INFRASTRUCTURE ONLY.

Format: the OCP Microscaling (MX) layout "MXFP4" (OCP Microscaling Formats specification v1.0,
2023): elements are FP4 E2M1 (1 sign, 2 exponent bits with bias 1, 1 mantissa bit; exponent field
0 holds the subnormal 0.5; no infinity, no NaN; values 0, 0.5, 1, 1.5, 2, 3, 4, 6), and every block
of 32 consecutive elements of a row shares one E8M0 scale (a power of two 2^(byte - 127)).  The
choice of the scale is this library's (the specification leaves it to the converter): the smallest
power of two s with max|block| <= 6 s, so no element saturates; byte >= 1; an all-zero block gets
byte 127.  Elements: the E2M1 value nearest to W / s, ties to the even code.  An extension on the
MI355X side, not part of the paper; written out from the format in numpy fp64, shares nothing with
the library's kernels.  Only tests, the smoke check and the benchmark's baseline leg may import it.

The library hands its bytes out in blocked orders; ``blocked_data`` / ``unblocked_data`` and
``blocked_scales`` / ``unblocked_scales`` restate them with numpy reshapes.
"""
from __future__ import annotations

import math

import numpy as np

BLOCK = 32
E2M1_MAX = 6.0


def value_of_code(code: int) -> float:
    sign = -1.0 if code & 0x8 else 1.0
    ex = (code >> 1) & 0x3
    man = code & 0x1
    if ex == 0:
        return sign * man * 0.5
    return sign * (1.0 + man / 2.0) * 2.0 ** (ex - 1)


def code_values() -> np.ndarray:
    return np.array([value_of_code(c) for c in range(16)], dtype=np.float64)


def scale_exponent(absmax: float) -> int:
    """n of the scale 2^n: the smallest with absmax <= 6 * 2^n; 0 for an all-zero block; >= -126."""
    if not absmax > 0.0:
        return 0
    n = math.ceil(math.log2(absmax / E2M1_MAX))
    while absmax > E2M1_MAX * 2.0 ** n:      # settle the rounding of log2 exactly
        n += 1
    while absmax <= E2M1_MAX * 2.0 ** (n - 1):
        n -= 1
    return max(n, -126)


def nearest_code(v: np.ndarray) -> np.ndarray:
    """Element-wise nearest E2M1 value of |v| <= 6, ties to the even code -> codes 0..15."""
    v = np.asarray(v, dtype=np.float64)
    grid = code_values()[:8]                          # 0 .. 6, ascending with the code
    a = np.abs(v)
    if a.size and a.max() > E2M1_MAX:
        raise ValueError("value beyond the e2m1 range")
    hi = np.minimum(np.searchsorted(grid, a, side="left"), 7)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - grid[lo], grid[hi] - a
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(take_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(v), code | 0x8, code).astype(np.uint8)


def quantize(w: np.ndarray):
    """w [E, rows, cols] (cols a multiple of 32) -> (codes uint8 [E, rows, cols] with values 0..15,
    scale bytes uint8 [E, rows, cols // 32])."""
    w = np.asarray(w, dtype=np.float64)
    E, rows, cols = w.shape
    assert cols % BLOCK == 0
    blocks = w.reshape(E, rows, cols // BLOCK, BLOCK)
    absmax = np.abs(blocks).max(axis=3)
    n = np.vectorize(scale_exponent, otypes=[np.int64])(absmax)
    codes = nearest_code(blocks / (2.0 ** n)[..., None]).reshape(E, rows, cols)
    return codes, (n + 127).astype(np.uint8)


def dequantize(codes: np.ndarray, scale_bytes: np.ndarray) -> np.ndarray:
    """-> float64 [E, rows, cols] = 2^(byte - 127) * value(code)."""
    E, rows, cols = codes.shape
    vals = code_values()[codes].reshape(E, rows, cols // BLOCK, BLOCK)
    s = 2.0 ** (scale_bytes.astype(np.float64) - 127.0)
    return (vals * s[..., None]).reshape(E, rows, cols)


def blocked_data(codes: np.ndarray) -> np.ndarray:
    """[E, rows, cols] codes -> [E, rows * cols / 2] bytes in the library's order: element (n, k) is
    nibble k % 2 (low first) of byte ((n//32)*(cols//64) + k//64)*1024 + (n%32)*32 + (k%64)//2."""
    E, rows, cols = codes.shape
    assert rows % 32 == 0 and cols % 64 == 0
    packed = (codes[:, :, 0::2] | (codes[:, :, 1::2] << 4)).astype(np.uint8)          # [E, rows, cols/2]
    return packed.reshape(E, rows // 32, 32, cols // 64, 32).transpose(0, 1, 3, 2, 4).reshape(E, rows * cols // 2)


def unblocked_data(qb: np.ndarray, rows: int, cols: int) -> np.ndarray:
    E = qb.shape[0]
    packed = qb.reshape(E, rows // 32, cols // 64, 32, 32).transpose(0, 1, 3, 2, 4).reshape(E, rows, cols // 2)
    codes = np.empty((E, rows, cols), dtype=np.uint8)
    codes[:, :, 0::2] = packed & 0xF
    codes[:, :, 1::2] = packed >> 4
    return codes


def scale_bytes_per_expert(rows: int, cols: int) -> int:
    return (rows // 32) * ((cols + 511) // 512) * 512


def blocked_scales(sb: np.ndarray, rows: int, cols: int, pad: int = 127) -> np.ndarray:
    """[E, rows, cols // 32] -> [E, scale_bytes_per_expert]: scale of (n, block b) at byte
    ((n//32)*ceil(cols/512) + b//16)*512 + (n%32)*16 + b%16; padding bytes = pad."""
    E = sb.shape[0]
    groups = (cols + 511) // 512
    full = np.full((E, rows, groups * 16), pad, dtype=np.uint8)
    full[:, :, :cols // 32] = sb
    return full.reshape(E, rows // 32, 32, groups, 16).transpose(0, 1, 3, 2, 4).reshape(E, -1)


def unblocked_scales(sbb: np.ndarray, rows: int, cols: int) -> np.ndarray:
    E = sbb.shape[0]
    groups = (cols + 511) // 512
    full = sbb.reshape(E, rows // 32, groups, 32, 16).transpose(0, 1, 3, 2, 4).reshape(E, rows, groups * 16)
    return full[:, :, :cols // 32]
