"""Pins of the 4-bit block-scaled quantisation oracle: facts of the published format, brute force,
hand-worked blocks, the scale rule at its boundaries, the layout formulas."""
import numpy as np
import pytest

from oracle import quant_mxfp4 as oq


def test_e2m1_values_are_the_published_ones():
    v = oq.code_values()
    assert list(v[:8]) == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]        # OCP MX v1.0, FP4 E2M1
    assert list(v[8:]) == [-0.0, -0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0]
    assert np.signbit(v[8])


def test_nearest_code_against_brute_force_and_ties():
    rng = np.random.default_rng(0)
    x = rng.uniform(-6, 6, 5000)
    grid = oq.code_values()[:8]
    got = oq.code_values()[oq.nearest_code(x)]
    for xi, gi in zip(x, got):
        assert abs(gi - xi) == np.abs(grid - abs(xi)).min()
        assert np.sign(gi) == np.sign(xi) or gi == 0
    # every midpoint goes to the even code: 0.25->0, 0.75->1, 1.25->1, 1.75->2, 2.5->2, 3.5->4, 5->4
    mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    assert list(oq.nearest_code(mids)) == [0, 2, 2, 4, 4, 6, 6]
    assert list(oq.nearest_code(-mids)) == [8, 10, 10, 12, 12, 14, 14]
    assert list(oq.nearest_code(grid)) == list(range(8))                   # grid values are fixed points


@pytest.mark.parametrize("absmax, n", [(6.0, 0), (6.0 * (1 + 2.0 ** -20), 1), (5.9, 0), (3.0, -1), (3.01, 0), (1.0, -2),
                                       (0.0, 0), (0.75, -3), (1e-3, -12), (48.0, 3), (1e-45, -126)])
def test_scale_is_the_smallest_power_of_two_that_fits(absmax, n):
    assert oq.scale_exponent(absmax) == n
    if absmax > 1e-30:
        assert absmax <= 6.0 * 2.0 ** n and absmax > 3.0 * 2.0 ** n


def test_hand_worked_block():
    # one block: max 5 -> scale 1 (5 <= 6); values / 1 rounded: 5 -> tie between 4 and 6 -> 4 (even code 6)
    w = np.zeros((1, 1, 32))
    w[0, 0, :6] = [5.0, -2.4, 0.3, 0.2, 1.3, -0.76]
    codes, sb = oq.quantize(w)
    assert sb[0, 0, 0] == 127
    assert list(codes[0, 0, :6]) == [6, 12, 1, 0, 3, 10]      # 4, -2, 0.5, 0, 1.5, -1
    back = oq.dequantize(codes, sb)
    assert list(back[0, 0, :6]) == [4.0, -2.0, 0.5, 0.0, 1.5, -1.0]
    # the same block 16 times smaller: scale byte 123, same codes
    codes2, sb2 = oq.quantize(w / 16)
    assert sb2[0, 0, 0] == 123 and np.array_equal(codes2, codes)
    # an all-zero block
    c0, s0 = oq.quantize(np.zeros((1, 1, 32)))
    assert s0[0, 0, 0] == 127 and not c0.any()


def test_roundtrip_error_bound_and_fixed_points():
    rng = np.random.default_rng(1)
    w = rng.standard_normal((3, 64, 128)) * np.array([1e-3, 1.0, 50.0]).reshape(3, 1, 1)
    codes, sb = oq.quantize(w)
    back = oq.dequantize(codes, sb)
    s = 2.0 ** (sb.astype(np.float64) - 127)
    err = np.abs(back - w).reshape(3, 64, 4, 32)
    # spacing of the grid is at most 2 s (between 4 and 6): error <= s; and <= |w| / 4 + s / 4 in general
    assert np.all(err <= s[..., None] + 1e-300)
    assert np.all(np.abs(back).reshape(3, 64, 4, 32).max(axis=3) <= 6 * s)
    c2, s2 = oq.quantize(back)
    assert np.array_equal(oq.dequantize(c2, s2), back)


def test_blocked_orders_are_the_stated_formulas_and_invertible():
    rng = np.random.default_rng(2)
    E, rows, cols = 2, 64, 640                       # cols not a multiple of 512: one padded scale group
    codes = rng.integers(0, 16, (E, rows, cols), dtype=np.uint8)
    qb = oq.blocked_data(codes)
    assert qb.shape == (E, rows * cols // 2)
    for _ in range(3000):
        e, n, k = rng.integers(E), rng.integers(rows), rng.integers(cols)
        byte = qb[e, ((n // 32) * (cols // 64) + k // 64) * 1024 + (n % 32) * 32 + (k % 64) // 2]
        assert ((byte >> (4 * (k % 2))) & 0xF) == codes[e, n, k]
    assert np.array_equal(oq.unblocked_data(qb, rows, cols), codes)
    sb = rng.integers(1, 255, (E, rows, cols // 32), dtype=np.uint8)
    sbb = oq.blocked_scales(sb, rows, cols)
    assert sbb.shape == (E, oq.scale_bytes_per_expert(rows, cols)) and oq.scale_bytes_per_expert(rows, cols) == 2 * 2 * 512
    groups = (cols + 511) // 512
    for _ in range(2000):
        e, n, b = rng.integers(E), rng.integers(rows), rng.integers(cols // 32)
        assert sbb[e, ((n // 32) * groups + b // 16) * 512 + (n % 32) * 16 + b % 16] == sb[e, n, b]
    assert np.array_equal(oq.unblocked_scales(sbb, rows, cols), sb)
