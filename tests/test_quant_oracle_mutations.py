"""The pins of the two quantisation oracles must be able to fail: each plausible mistake is planted
in a copy of the oracle's source (on the CPU), the copy is loaded as a module, and the oracle's own
pin tests are run against it -- at least one of them has to fail."""
import inspect
import os
import types

import pytest

import test_quant_mxfp4_oracle as pins4
import test_quant_oracle as pins8

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = {
    # name: (oracle file, pin module, text to replace, replacement)
    "e4m3_bias": ("quant_e4m3.py", pins8, "2.0 ** (ex - 7)", "2.0 ** (ex - 8)"),
    "e4m3_subnormal_scale": ("quant_e4m3.py", pins8, "(man / 8.0) * 2.0 ** -6", "(man / 8.0) * 2.0 ** -7"),
    "e4m3_ties_to_odd": ("quant_e4m3.py", pins8, "((d_hi == d_lo) & (hi % 2 == 0))", "((d_hi == d_lo) & (hi % 2 == 1))"),
    "e4m3_round_down": ("quant_e4m3.py", pins8, "take_hi = (d_hi < d_lo) |", "take_hi = (d_hi < d_lo) & (d_hi < 0) |"),
    "e4m3_scale_one_too_large": ("quant_e4m3.py", pins8, "return 2.0 ** max(n, -126)", "return 2.0 ** max(n + 1, -126)"),
    "e4m3_sign_dropped": ("quant_e4m3.py", pins8, "return np.where(neg, code | 0x80, code).astype(np.uint8)",
                          "return code.astype(np.uint8)"),
    "e4m3_blocked_rows_and_cols_swapped": ("quant_e4m3.py", pins8,
                                           "q.reshape(E, rows // 16, 16, cols // 64, 64).transpose(0, 1, 3, 2, 4)",
                                           "q.reshape(E, rows // 16, 16, cols // 64, 64).transpose(0, 3, 1, 2, 4)"),
    "mxfp4_value_table": ("quant_mxfp4.py", pins4, "return sign * (1.0 + man / 2.0) * 2.0 ** (ex - 1)",
                          "return sign * (1.0 + man / 2.0) * 2.0 ** ex"),
    "mxfp4_ties_to_odd": ("quant_mxfp4.py", pins4, "((d_hi == d_lo) & (hi % 2 == 0))", "((d_hi == d_lo) & (hi % 2 == 1))"),
    "mxfp4_scale_floor_rule": ("quant_mxfp4.py", pins4, "return max(n, -126)", "return max(n - 1, -126)"),
    "mxfp4_block_of_16": ("quant_mxfp4.py", pins4, "BLOCK = 32", "BLOCK = 16"),
    "mxfp4_high_nibble_first": ("quant_mxfp4.py", pins4, "(codes[:, :, 0::2] | (codes[:, :, 1::2] << 4))",
                                "(codes[:, :, 1::2] | (codes[:, :, 0::2] << 4))"),
    "mxfp4_scale_byte_bias": ("quant_mxfp4.py", pins4, "return codes, (n + 127).astype(np.uint8)",
                              "return codes, (n + 128).astype(np.uint8)"),
    "mxfp4_scales_row_major": ("quant_mxfp4.py", pins4,
                               "full.reshape(E, rows // 32, 32, groups, 16).transpose(0, 1, 3, 2, 4).reshape(E, -1)",
                               "full.reshape(E, -1)"),
}


def load_mutant(name):
    fname, pins, old, new = MUTATIONS[name]
    text = open(os.path.join(ROOT, "oracle", fname)).read()
    assert text.count(old) >= 1, "mutation site for %s not found" % name
    mod = types.ModuleType("mutant_" + name)
    exec(compile(text.replace(old, new, 1), fname, "exec"), mod.__dict__)
    return mod, pins


def run_pins(pins, oracle):
    """Run every test function of the pin module against `oracle`; return the names of those that fail."""
    saved = pins.oq
    pins.oq = oracle
    failed = []
    try:
        for fname, fn in inspect.getmembers(pins, inspect.isfunction):
            if not fname.startswith("test_"):
                continue
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            arg_sets = [()]
            if marks:
                arg_sets = [a if isinstance(a, tuple) else (a,) for a in marks[0].args[1]]
            for args in arg_sets:
                try:
                    fn(*args)
                except Exception:  # an assertion, or the mutant breaking down altogether
                    failed.append(fname)
                    break
    finally:
        pins.oq = saved
    return failed


def test_pins_pass_on_the_unmodified_oracles():
    from oracle import quant_e4m3, quant_mxfp4
    assert run_pins(pins8, quant_e4m3) == []
    assert run_pins(pins4, quant_mxfp4) == []


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name):
    mod, pins = load_mutant(name)
    assert run_pins(pins, mod), "no pin noticed the planted mistake '%s'" % name
