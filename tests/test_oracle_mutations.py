"""The oracle's pins must be able to fail: each plausible mistake is planted in a COPY of
oracle/moe_oracle.c (on the CPU, never in the GPU path), the copy is compiled, and the pin that
is meant to catch that kind of mistake is run against it and has to report a mismatch."""
import ctypes
import os
import subprocess

import numpy as np
import pytest
import scipy.special

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "moe_oracle.c")

MUTATIONS = {
    # name: (text to replace, replacement)
    "tie_to_highest_index": ("if (best < 0 || l[e] > l[best])", "if (best < 0 || l[e] >= l[best])"),
    "topk_smallest": ("if (best < 0 || l[e] > l[best])", "if (best < 0 || l[e] < l[best])"),
    "softmax_sign": ("w[(size_t)t * k + j] = exp((double)l[sel[j]] - m) / denom;",
                     "w[(size_t)t * k + j] = exp(m - (double)l[sel[j]]) / denom;"),
    "gate_bias_dropped": ("acc += (double)bias[e];", "acc += 0.0;"),
    "offsets_off_by_one": ("offsets[e + 1] = offsets[e] + counts[e];", "offsets[e + 1] = offsets[e] + counts[e] + (e == 0);"),
    "rank_not_stable": ("int r = offsets[e] + seen[e];", "int r = offsets[e] + (counts[e] - 1 - seen[e]);"),
    "relu_dropped": ("h[f] = acc > 0.0 ? acc : 0.0;", "h[f] = acc;"),
    "w2_transposed": ("size_t base = ((size_t)e * D + d) * F;", "size_t base = ((size_t)e * D) * F + d;"),
    "gate_weight_dropped": ("yr[d] += g * o[d];", "yr[d] += o[d];"),
    "b2_dropped": ("acc += ld(b2, (size_t)e * D + d, dt);", "acc += 0.0;"),
    "static_second_choice_first": ("for (int j = 0; j < k; ++j) {\n        for (int t = 0; t < T; ++t) {",
                                   "for (int j = k - 1; j >= 0; --j) {\n        for (int t = 0; t < T; ++t) {"),
    "static_capacity_off_by_one": ("if (fill[e] < capacity) {", "if (fill[e] <= capacity) {"),
    "b1_dropped": ("acc += ld(b1, (size_t)e * F + f, dt);", "acc += 0.0;"),
    "renormalisation_ignored": ("        if (renorm) {\n            for (int j = 0; j < k; ++j)", "        if (0) {\n            for (int j = 0; j < k; ++j)"),
    "raw_softmax_renormalised": ("            for (int e = 0; e < E; ++e)\n                denom += exp((double)l[e] - m);",
                                 "            for (int j = 0; j < k; ++j)\n                denom += exp((double)l[sel[j]] - m);"),
    "w1_transposed": ("size_t base = ((size_t)e * F + f) * D;", "size_t base = ((size_t)e * F) * D + f;"),
}


def build_mutant(tmp_path, name):
    text = open(SRC).read()
    old, new = MUTATIONS[name]
    assert text.count(old) >= 1, "mutation site for %s not found" % name
    text = text.replace(old, new, 1)
    c = tmp_path / (name + ".c")
    so = tmp_path / (name + ".so")
    c.write_text(text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    lib.moe_oracle_route.restype = ctypes.c_int
    lib.moe_oracle_static_slots.restype = ctypes.c_int
    return lib


def P(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def rnd(seed, *shape, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


# ---- the pins, written against a raw library handle -------------------------------------------
def pin_topk(lib):
    l = rnd(1, 30, 9)
    l[2, :] = 0.5
    l[3, 4] = l[3, 7] = 9.0
    T, E, k = l.shape[0], l.shape[1], 2
    idx = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float64)
    lib.moe_oracle_topk(P(l), T, E, k, 1, P(idx), P(w))
    ref = np.array([sorted(range(E), key=lambda e: (-float(l[t, e]), e))[:k] for t in range(T)], np.int32)
    p = scipy.special.softmax(l.astype(np.float64), axis=1)
    p2 = np.take_along_axis(p, ref.astype(np.int64), 1)
    ok = np.array_equal(idx, ref) and np.allclose(w, p2 / p2.sum(1, keepdims=True), rtol=1e-12)
    # without renormalisation the weights are the softmax probabilities themselves
    lib.moe_oracle_topk(P(l), T, E, k, 0, P(idx), P(w))
    return ok and np.array_equal(idx, ref) and np.allclose(w, p2, rtol=1e-12)


def pin_logits(lib):
    x, wg, b = rnd(2, 11, 16), rnd(3, 5, 16), rnd(4, 5)
    out = np.empty((11, 5), np.float32)
    lib.moe_oracle_gate_logits(P(x), P(wg), P(b), 11, 16, 5, 0, P(out))
    ref = (x.astype(np.float64) @ wg.astype(np.float64).T + b).astype(np.float32)
    return np.array_equal(out, ref)


def pin_route(lib):
    rng = np.random.default_rng(5)
    T, E, k = 200, 7, 2
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    counts, offsets = np.empty(E, np.int32), np.empty(E + 1, np.int32)
    dst, src = np.empty((T, k), np.int32), np.empty(T * k, np.int32)
    lib.moe_oracle_route(P(idx), T, E, k, P(counts), P(offsets), P(dst), P(src))
    order = np.argsort(idx.ravel(), kind="stable")
    inv = np.empty(T * k, np.int64)
    inv[order] = np.arange(T * k)
    return (np.array_equal(counts, np.bincount(idx.ravel(), minlength=E)) and offsets[E] == T * k
            and np.array_equal(src, order // k) and np.array_equal(dst.ravel(), inv))


def pin_layer(lib):
    T, D, F, E, k = 17, 8, 12, 4, 2
    x, w1, w2 = rnd(6, T, D), rnd(7, E, F, D), rnd(8, E, D, F)
    b1, b2 = rnd(9, E, F), rnd(10, E, D)
    rng = np.random.default_rng(11)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    w = rng.random((T, k))
    y = np.empty((T, D), np.float64)
    lib.moe_oracle_layer_tokens(P(x), P(w1), P(w2), P(b1), P(b2), P(idx), P(w), None, None, T, D, F, k, 0, P(y))
    ref = np.zeros((T, D))
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            h = np.maximum(w1[e].astype(np.float64) @ x[t].astype(np.float64) + b1[e], 0)
            ref[t] += w[t, j] * (w2[e].astype(np.float64) @ h + b2[e])
    return np.allclose(y, ref, rtol=1e-11, atol=1e-12)


def pin_static(lib):
    idx = np.array([[1, 0], [1, 0], [0, 1], [0, 2], [0, 1]], np.int32)
    slot, keep = np.empty((5, 2), np.int32), np.empty((5, 2), np.uint8)
    dropped = lib.moe_oracle_static_slots(P(idx), 5, 3, 2, 2, P(slot), P(keep))
    return dropped == 5 and np.array_equal(slot, [[0, -1], [1, -1], [0, -1], [1, 0], [-1, -1]])


CATCHES = {
    "tie_to_highest_index": pin_topk, "topk_smallest": pin_topk, "softmax_sign": pin_topk,
    "gate_bias_dropped": pin_logits,
    "offsets_off_by_one": pin_route, "rank_not_stable": pin_route,
    "relu_dropped": pin_layer, "w2_transposed": pin_layer, "gate_weight_dropped": pin_layer, "b2_dropped": pin_layer,
    "static_second_choice_first": pin_static, "static_capacity_off_by_one": pin_static,
    "b1_dropped": pin_layer, "w1_transposed": pin_layer,
    "renormalisation_ignored": pin_topk, "raw_softmax_renormalised": pin_topk,
}


def test_pins_pass_on_the_unmodified_oracle(tmp_path):
    text = open(SRC).read()
    c = tmp_path / "orig.c"
    so = tmp_path / "orig.so"
    c.write_text(text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    lib.moe_oracle_route.restype = ctypes.c_int
    lib.moe_oracle_static_slots.restype = ctypes.c_int
    for pin in (pin_topk, pin_logits, pin_route, pin_layer, pin_static):
        assert pin(lib), pin.__name__


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, name):
    lib = build_mutant(tmp_path, name)
    assert not CATCHES[name](lib), "the pin did not notice the planted mistake '%s'" % name
