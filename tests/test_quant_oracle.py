"""Pins of the e4m3 quantisation oracle: facts of the published format, PyTorch's own
float8_e4m3fn conversion (a library routine written by others), and brute force."""
import numpy as np
import pytest
import torch

from oracle import quant_e4m3 as oq


def test_format_facts():
    v = oq.code_values()
    assert v[0x7E] == 448.0 and v[0xFE] == -448.0           # largest finite
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF])          # the only NaN codes, no infinity
    assert v[0x01] == 2.0 ** -9                             # smallest subnormal
    assert v[0x08] == 2.0 ** -6                             # smallest normal
    assert v[0x38] == 1.0 and v[0x39] == 1.125              # bias 7, 3 mantissa bits
    assert v[0x00] == 0.0 and v[0x80] == 0.0 and np.signbit(v[0x80])
    assert np.all(np.diff(v[:0x7F]) > 0)                    # non-negative codes ascend with value


def test_code_values_equal_torch_float8_e4m3fn():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    t = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    v = oq.code_values()
    nan = np.isnan(v)
    assert np.array_equal(nan, np.isnan(t))
    assert np.array_equal(v[~nan], t[~nan])


def test_nearest_code_equals_torch_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.uniform(-448, 448, 20000), rng.standard_normal(20000), rng.standard_normal(20000) * 2.0 ** -7,
        oq.code_values()[:0x7F],                                             # every grid value
        (oq.code_values()[:0x7E] + oq.code_values()[1:0x7F]) / 2,            # every midpoint: ties
        -(oq.code_values()[:0x7E] + oq.code_values()[1:0x7F]) / 2,
    ]).astype(np.float32)
    got = oq.nearest_code(x.astype(np.float64))
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    # -0 and +0 are the same number; compare values and, for non-zero inputs, the bytes
    nz = x != 0
    assert np.array_equal(got[nz], ref[nz])
    assert np.all(oq.code_values()[got[~nz]] == 0)


def test_nearest_code_against_brute_force():
    rng = np.random.default_rng(1)
    x = rng.uniform(-448, 448, 3000)
    x[:500] *= 2.0 ** -10
    grid = oq.code_values()[:0x7F]
    got = oq.code_values()[oq.nearest_code(x)]
    for xi, gi in zip(x, got):
        assert abs(gi - xi) == np.abs(grid - abs(xi)).min()
        assert np.sign(gi) == np.sign(xi) or gi == 0


def test_ties_go_to_the_even_mantissa():
    assert oq.nearest_code(np.array([1.0625]))[0] == 0x38      # between 1.0 (m=0) and 1.125 (m=1)
    assert oq.nearest_code(np.array([1.1875]))[0] == 0x3A      # between 1.125 (m=1) and 1.25 (m=2)
    assert oq.nearest_code(np.array([2.0 ** -10]))[0] == 0x00  # between 0 and the smallest subnormal
    assert oq.nearest_code(np.array([-3 * 2.0 ** -10]))[0] == 0x82


@pytest.mark.parametrize("absmax, want", [
    (448.0, 1.0), (448.0 * (1 + 2.0 ** -20), 2.0), (447.0, 1.0), (224.0, 0.5), (224.5, 1.0), (1.0, 2.0 ** -8),
    (0.0, 1.0), (7.0, 2.0 ** -6), (7.0 * (1 + 2.0 ** -23), 2.0 ** -5), (1e-3, 2.0 ** -18), (3e4, 128.0),
])
def test_scale_is_the_smallest_power_of_two_that_fits(absmax, want):
    s = oq.scale_of(absmax)
    assert s == want
    if absmax > 0:
        assert absmax <= 448.0 * s and absmax > 448.0 * s / 2


def test_quantize_roundtrip_error_bound_and_fixed_points():
    rng = np.random.default_rng(2)
    w = rng.standard_normal((5, 64, 48)) * np.array([1e-3, 0.02, 1.0, 30.0, 0.0]).reshape(5, 1, 1)
    q, s = oq.quantize(w)
    back = oq.dequantize(q, s)
    assert s[4] == 1.0 and np.all(back[4] == 0)
    for e in range(4):
        # normal range: relative error <= 2^-4; below the smallest normal: absolute error <= 2^-10 s
        err = np.abs(back[e] - w[e])
        assert np.all(err <= np.maximum(np.abs(w[e]) * 2.0 ** -4, s[e] * 2.0 ** -10))
        assert np.abs(back[e]).max() <= 448.0 * s[e]
    # values already on the grid come back unchanged
    q2, s2 = oq.quantize(back[:4])
    assert np.array_equal(oq.dequantize(q2, s2), back[:4])


def test_blocked_order_is_the_stated_formula_and_invertible():
    rng = np.random.default_rng(3)
    E, rows, cols = 3, 48, 192
    q = rng.integers(0, 256, (E, rows, cols), dtype=np.uint8)
    b = oq.blocked(q)
    for _ in range(2000):
        e, n, k = rng.integers(E), rng.integers(rows), rng.integers(cols)
        assert b[e, ((n // 16) * (cols // 64) + k // 64) * 1024 + (n % 16) * 64 + k % 64] == q[e, n, k]
    assert np.array_equal(oq.unblocked(b, rows, cols), q)
