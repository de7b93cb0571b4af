"""Pins for the CPU oracle: it is checked against things other than itself --
the paper's worked example and closed forms (tests/golden), textbook routines
(numpy matmul, scipy softmax, numpy stable argsort + bincount), a dense brute-force
formulation, and invariants the paper's definitions fix.  No GPU is used here."""
import json
import os

import numpy as np
import pytest
import scipy.special
import torch

from paper_2303_06182_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(seed, *shape, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def small_layer(seed=0, T=37, D=24, F=40, E=5, gate_scale=3.0):
    x = rnd(seed, T, D)
    wg = rnd(seed + 1, E, D, scale=gate_scale / np.sqrt(D))
    w1 = rnd(seed + 2, E, F, D, scale=0.3)
    w2 = rnd(seed + 3, E, D, F, scale=0.3)
    return x, wg, w1, w2


def np_ffn(x64, w1e, w2e, b1e=None, b2e=None):
    h = x64 @ w1e.astype(np.float64).T
    if b1e is not None:
        h = h + b1e.astype(np.float64)
    h = np.maximum(h, 0.0)
    o = h @ w2e.astype(np.float64).T
    if b2e is not None:
        o = o + b2e.astype(np.float64)
    return o


# ----------------------------------------------------------------------------- gate
def test_gate_logits_match_numpy_matmul(oracle):
    x = rnd(1, 19, 33)
    wg = rnd(2, 7, 33)
    bias = rnd(3, 7)
    ref = x.astype(np.float64) @ wg.astype(np.float64).T + bias.astype(np.float64)
    got = oracle.gate_logits(x, wg, bias)
    assert got.dtype == np.float32 and got.shape == (19, 7)
    np.testing.assert_array_equal(got, ref.astype(np.float32))
    np.testing.assert_array_equal(oracle.gate_logits(x, wg), (ref - bias).astype(np.float32))


def test_gate_logits_bf16_storage_is_exact_widening(oracle):
    x = torch.from_numpy(rnd(4, 11, 16)).to(torch.bfloat16)
    wg = torch.from_numpy(rnd(5, 6, 16)).to(torch.bfloat16)
    a = oracle.gate_logits(x, wg)
    b = oracle.gate_logits(x.float(), wg.float())
    np.testing.assert_array_equal(a, b)


# ----------------------------------------------------------------------------- top-k
def brute_topk(l, k):
    T, E = l.shape
    out = np.empty((T, k), dtype=np.int32)
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-float(l[t, e]), e))
        out[t] = order[:k]
    return out


@pytest.mark.parametrize("E,k", [(8, 2), (5, 1), (13, 3), (64, 2), (128, 2), (6, 6)])
def test_topk_matches_brute_force(oracle, E, k):
    l = rnd(E * 10 + k, 50, E)
    l[3, :] = 0.25                       # an all-equal row
    l[4, : E // 2] = l[4, E // 2: 2 * (E // 2)]  # pairs of equal values
    idx, w = oracle.topk(l, k)
    np.testing.assert_array_equal(idx, brute_topk(l, k))
    for t in range(l.shape[0]):
        assert len(set(idx[t])) == k


def test_topk_ties_go_to_lowest_index(oracle):
    l = np.zeros((3, 12), dtype=np.float32)
    l[1, 5] = l[1, 9] = 2.0          # duplicated maximum at 5 and 9
    l[2, 11] = 1.0
    l[2, 0] = l[2, 7] = 0.5
    idx, w = oracle.topk(l, 2)
    np.testing.assert_array_equal(idx, [[0, 1], [5, 9], [11, 0]])
    np.testing.assert_allclose(w[0], [0.5, 0.5])
    np.testing.assert_allclose(w[1], [0.5, 0.5])


def test_gate_weights_are_the_softmax(oracle):
    l = rnd(7, 40, 9, scale=2.0)
    p = scipy.special.softmax(l.astype(np.float64), axis=1)
    # k = E: all experts selected, ordered by logit; weights = textbook softmax
    idx, w = oracle.topk(l, 9)
    np.testing.assert_allclose(w, np.take_along_axis(p, idx.astype(np.int64), 1), rtol=1e-13)
    assert np.all(np.diff(np.take_along_axis(l, idx.astype(np.int64), 1), axis=1) <= 0)
    # k = 1: weight 1
    idx1, w1 = oracle.topk(l, 1)
    np.testing.assert_array_equal(w1, 1.0)
    np.testing.assert_array_equal(idx1[:, 0], np.argmax(l, axis=1))
    # top-2 renormalised: ratio of softmax probabilities, sums to 1
    idx2, w2 = oracle.topk(l, 2)
    p2 = np.take_along_axis(p, idx2.astype(np.int64), 1)
    np.testing.assert_allclose(w2, p2 / p2.sum(1, keepdims=True), rtol=1e-13)
    np.testing.assert_allclose(w2.sum(1), 1.0, rtol=1e-14)
    assert np.all(w2[:, 0] >= w2[:, 1])
    # not renormalised: the raw probabilities
    _, w2r = oracle.topk(l, 2, renormalize=False)
    np.testing.assert_allclose(w2r, p2, rtol=1e-13)


# ----------------------------------------------------------------------------- routing
def check_route_invariants(idx, E, counts, offsets, dst_row, src_tok):
    T, k = idx.shape
    N = T * k
    assert counts.sum() == N                                  # every assignment counted once
    assert offsets[0] == 0 and offsets[E] == N
    np.testing.assert_array_equal(np.diff(offsets), counts)
    assert sorted(dst_row.ravel().tolist()) == list(range(N))  # bijection: nothing dropped, no padding
    for t in range(T):
        for j in range(k):
            r = dst_row[t, j]
            assert src_tok[r] == t
            e = idx[t, j]
            assert offsets[e] <= r < offsets[e + 1]           # the row sits in its expert's range
    for e in range(E):
        seg = src_tok[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(seg) > 0)                       # ascending token order, no repeats


@pytest.mark.parametrize("T,E,k,seed", [(1, 4, 2, 0), (64, 8, 2, 1), (300, 16, 2, 2), (97, 128, 2, 3),
                                        (200, 7, 3, 4), (50, 3, 1, 5)])
def test_route_invariants_and_argsort_form(oracle, T, E, k, seed):
    l = rnd(seed, T, E)
    idx, _ = oracle.topk(l, k)
    counts, offsets, dst_row, src_tok = oracle.route(idx, E)
    check_route_invariants(idx, E, counts, offsets, dst_row, src_tok)
    # the paper's own formulation: a (stable) argsort of the flat expert assignment and a bin count
    flat = idx.ravel()                      # assignment a = t*k + j
    order = np.argsort(flat, kind="stable")
    np.testing.assert_array_equal(counts, np.bincount(flat, minlength=E))
    # a token never picks an expert twice, so sorting by (expert, t*k+j) == by (expert, t)
    np.testing.assert_array_equal(src_tok, order // k)
    inv = np.empty(T * k, dtype=np.int64)
    inv[order] = np.arange(T * k)
    np.testing.assert_array_equal(dst_row.ravel(), inv)


def test_route_empty_experts_and_bad_index(oracle):
    idx = np.array([[2, 5], [5, 2], [2, 7]], dtype=np.int32)
    counts, offsets, dst_row, src_tok = oracle.route(idx, 9)
    np.testing.assert_array_equal(counts, [0, 0, 3, 0, 0, 2, 0, 1, 0])
    np.testing.assert_array_equal(offsets, [0, 0, 0, 3, 3, 3, 5, 5, 6, 6])
    np.testing.assert_array_equal(dst_row, [[0, 3], [4, 1], [2, 5]])
    np.testing.assert_array_equal(src_tok, [0, 1, 2, 0, 1, 2])
    with pytest.raises(ValueError):
        oracle.route(np.array([[0, 9]], dtype=np.int32), 9)


# ----------------------------------------------------------------------------- layer output
def dense_brute_force(x, wg, w1, w2, k, bias=None, b1=None, b2=None, renorm=True):
    """Second formulation: run EVERY expert on EVERY token, then weight by the gate."""
    x64 = x.astype(np.float64)
    T, E = x.shape[0], wg.shape[0]
    logits = (x64 @ wg.astype(np.float64).T + (0 if bias is None else bias.astype(np.float64))).astype(np.float32)
    allout = np.stack([np_ffn(x64, w1[e], w2[e], None if b1 is None else b1[e], None if b2 is None else b2[e])
                       for e in range(E)])          # [E,T,D]
    y = np.zeros_like(x64)
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-float(logits[t, e]), e))[:k]
        p = scipy.special.softmax(logits[t].astype(np.float64))
        g = {e: p[e] for e in order}
        s = sum(g.values()) if renorm else 1.0
        for e in range(E):
            if e in g:
                y[t] += (g[e] / s) * allout[e, t]
    return y


@pytest.mark.parametrize("k,renorm,with_bias", [(2, True, False), (1, True, False), (3, False, True), (2, True, True)])
def test_layer_equals_dense_brute_force(oracle, k, renorm, with_bias):
    x, wg, w1, w2 = small_layer(seed=10 + k)
    E, F, D = w1.shape
    bias = rnd(90, E) if with_bias else None
    b1 = rnd(91, E, F, scale=0.2) if with_bias else None
    b2 = rnd(92, E, D, scale=0.2) if with_bias else None
    r = oracle.layer(x, wg, w1, w2, k, gate_bias=bias, b1=b1, b2=b2, renormalize=renorm)
    ref = dense_brute_force(x, wg, w1, w2, k, bias, b1, b2, renorm)
    np.testing.assert_allclose(r["y"], ref, rtol=1e-11, atol=1e-12)


def test_single_expert_is_a_plain_mlp(oracle):
    x, _, w1, w2 = small_layer(seed=20, E=1, T=23, D=32, F=48)
    wg = rnd(21, 1, 32)
    r = oracle.layer(x, wg, w1, w2, 1)
    ref = (torch.relu(torch.from_numpy(x).double() @ torch.from_numpy(w1[0]).double().T)
           @ torch.from_numpy(w2[0]).double().T).numpy()
    np.testing.assert_allclose(r["y"], ref, rtol=1e-12, atol=1e-13)
    assert np.all(r["idx"] == 0) and np.all(r["w"] == 1.0)


def test_identical_experts_give_the_dense_ffn(oracle):
    x, wg, w1, w2 = small_layer(seed=30)
    w1[:] = w1[0]
    w2[:] = w2[0]
    r = oracle.layer(x, wg, w1, w2, 2)
    np.testing.assert_allclose(r["y"], np_ffn(x.astype(np.float64), w1[0], w2[0]), rtol=1e-11, atol=1e-12)


def test_token_permutation_and_expert_relabelling(oracle):
    x, wg, w1, w2 = small_layer(seed=40)
    r = oracle.layer(x, wg, w1, w2, 2)
    p = np.random.default_rng(0).permutation(x.shape[0])
    rp = oracle.layer(x[p], wg, w1, w2, 2)
    np.testing.assert_array_equal(rp["y"], r["y"][p])
    np.testing.assert_array_equal(rp["idx"], r["idx"][p])
    q = np.random.default_rng(1).permutation(wg.shape[0])     # new expert i is old expert q[i]
    rq = oracle.layer(x, wg[q], w1[q], w2[q], 2)
    np.testing.assert_array_equal(q[rq["idx"]], r["idx"])
    np.testing.assert_array_equal(rq["y"], r["y"])


def test_idle_experts_never_touch_the_output(oracle):
    x, wg, w1, w2 = small_layer(seed=50, E=6)
    bias = np.array([0, -1e3, 0, -1e3, 0, 0], dtype=np.float32)   # experts 1 and 3 never win
    r = oracle.layer(x, wg, w1, w2, 2, gate_bias=bias)
    assert r["counts"][1] == 0 and r["counts"][3] == 0
    w1n, w2n = w1.copy(), w2.copy()
    w1n[[1, 3]] = np.nan
    w2n[[1, 3]] = np.nan
    rn = oracle.layer(x, wg, w1n, w2n, 2, gate_bias=bias)
    assert np.all(np.isfinite(rn["y"]))
    np.testing.assert_array_equal(rn["y"], r["y"])


def test_stage_functions_compose_to_the_layer(oracle):
    """dispatch -> grouped FFN -> combine (the dynamic-gating data path) equals the
    per-token definition; dispatch and combine are checked against explicit loops."""
    x, wg, w1, w2 = small_layer(seed=60)
    r = oracle.layer(x, wg, w1, w2, 2)
    xp = oracle.dispatch(x, r["src_tok"])
    for row in range(xp.shape[0]):
        np.testing.assert_array_equal(xp[row], x[r["src_tok"][row]].astype(np.float64))
    yp = oracle.expert_ffn(xp.astype(np.float32), r["offsets"], w1, w2)
    for e in range(wg.shape[0]):
        a, b = r["offsets"][e], r["offsets"][e + 1]
        np.testing.assert_allclose(yp[a:b], np_ffn(xp[a:b], w1[e], w2[e]), rtol=1e-11, atol=1e-12)
    y = oracle.combine(yp, r["dst_row"], r["w"])
    yl = np.zeros_like(y)
    for t in range(x.shape[0]):
        for j in range(2):
            yl[t] += r["w"][t, j] * yp[r["dst_row"][t, j]]
    np.testing.assert_allclose(y, yl, rtol=1e-14)
    np.testing.assert_allclose(y, r["y"], rtol=1e-11, atol=1e-13)
    # a sample of rows / tokens gives the same rows as the full computation
    rows = [0, 5, xp.shape[0] - 1]
    np.testing.assert_array_equal(oracle.expert_ffn(xp.astype(np.float32), r["offsets"], w1, w2, rows=rows), yp[rows])
    toks = [3, 36, 0]
    np.testing.assert_array_equal(oracle.layer_tokens(x, w1, w2, r["idx"], r["w"], tokens=toks), r["y"][toks])


def test_bf16_storage_equals_fp32_storage_of_the_same_values(oracle):
    x, wg, w1, w2 = small_layer(seed=70)
    tb = [torch.from_numpy(a).to(torch.bfloat16) for a in (x, wg, w1, w2)]
    a = oracle.layer(*tb, 2)
    b = oracle.layer(*[t.float() for t in tb], 2)
    np.testing.assert_array_equal(a["idx"], b["idx"])
    np.testing.assert_array_equal(a["y"], b["y"])


# ----------------------------------------------------------------------------- static gating
def test_static_example_from_the_paper(oracle):
    g = json.load(open(os.path.join(GOLDEN, "static_gating_example.json")))
    S, E, C = g["S"], g["E"], g["C"]
    cap = oracle.capacity_paper(C, S)
    assert cap == g["capacity"]
    idx = np.array(g["assignment"], dtype=np.int32).reshape(S, 1)
    slot, keep, dropped = oracle.static_slots(idx, E, cap)
    np.testing.assert_array_equal(slot[:, 0], g["expected_slot"])
    assert dropped == len(g["expected_dropped_tokens"])
    assert [t for t in range(S) if not keep[t, 0]] == g["expected_dropped_tokens"]
    mask, cw = oracle.static_masks(idx, np.ones((S, 1)), E, cap)
    assert list(mask.shape) == g["mask_shape"]
    assert mask.sum() == g["expected_ones_in_mask"] <= S          # at most S ones
    used = mask.sum(axis=(1, 2)).astype(int).tolist()
    assert used == g["expected_rows_used"]
    assert [cap - u for u in used] == g["expected_empty_rows"]
    assert np.all(mask.sum(axis=1) <= 1)      # a row holds at most one token
    assert np.all(mask.sum(axis=2) <= 1)      # a (token, expert) pair uses at most one row
    # the dropped token's output row is zero; every other row is its expert's FFN output
    D, F = 8, 12
    x = rnd(80, S, D)
    w1 = rnd(81, E, F, D)
    w2 = rnd(82, E, D, F)
    wts = np.ones((S, 1))
    y = oracle.layer_tokens(x, w1, w2, idx, wts, keep=keep)
    for t in range(S):
        if t in g["expected_dropped_tokens"]:
            assert np.all(y[t] == 0.0)
        else:
            np.testing.assert_allclose(y[t], np_ffn(x[t].astype(np.float64), w1[idx[t, 0]], w2[idx[t, 0]]),
                                       rtol=1e-12, atol=1e-13)


def test_waste_factors_from_the_paper(oracle):
    g = json.load(open(os.path.join(GOLDEN, "waste_factors.json")))
    for c in g["cases"]:
        S = 4000
        cap = oracle.capacity_paper(c["C"], S)
        assert cap * c["E"] / S == pytest.approx(c["rows_per_S"])
        assert cap * c["E"] / (c["k"] * S) == pytest.approx(c["waste_factor"])


def static_einsum_layer(x, w1, w2, idx, w, E, cap, oracle):
    """The paper's static data path written with dense masks: dispatch = mask x tokens,
    experts on `cap` rows each (zero rows included), combine = weights x expert outputs."""
    mask, cw = oracle.static_masks(idx, w, E, cap)
    xd = np.einsum("esc,sd->ecd", mask, x.astype(np.float64))
    yd = np.stack([np_ffn(xd[e], w1[e], w2[e]) for e in range(E)])
    return np.einsum("esc,ecd->sd", cw, yd)


@pytest.mark.parametrize("cap", [2, 5, 9, 40])
def test_static_index_form_equals_mask_form(oracle, cap):
    x, wg, w1, w2 = small_layer(seed=100)
    E = wg.shape[0]
    r = oracle.static_layer(x, wg, w1, w2, 2, cap)
    ref = static_einsum_layer(x, w1, w2, r["idx"], r["w"], E, cap, oracle)
    np.testing.assert_allclose(r["y"], ref, rtol=1e-11, atol=1e-12)
    assert r["dropped"] == int((r["keep"] == 0).sum())
    fill = np.zeros(E, dtype=int)
    for t in range(x.shape[0]):
        for j in range(2):
            if r["keep"][t, j]:
                fill[r["idx"][t, j]] += 1
    assert fill.max() <= cap


def test_static_equals_dynamic_when_nothing_is_dropped(oracle):
    x, wg, w1, w2 = small_layer(seed=110)
    dyn = oracle.layer(x, wg, w1, w2, 2)
    cap = int(dyn["counts"].max())
    st = oracle.static_layer(x, wg, w1, w2, 2, cap)
    assert st["dropped"] == 0
    np.testing.assert_array_equal(st["y"], dyn["y"])
    st_small = oracle.static_layer(x, wg, w1, w2, 2, cap - 1)
    assert st_small["dropped"] >= 1
    assert not np.array_equal(st_small["y"], dyn["y"])


def test_static_first_choices_fill_before_second_choices(oracle):
    # tokens 0..3; expert 0 is the SECOND choice of tokens 0,1 and the FIRST choice of tokens 2,3
    idx = np.array([[1, 0], [1, 0], [0, 1], [0, 2]], dtype=np.int32)
    slot, keep, dropped = oracle.static_slots(idx, 3, 2)
    np.testing.assert_array_equal(slot, [[0, -1], [1, -1], [0, -1], [1, 0]])
    assert dropped == 3


def test_capacity_conventions(oracle):
    assert oracle.capacity_paper(0.5, 6) == 3
    assert oracle.capacity_share(1.0, 65536, 128, 2) == 1024
    assert oracle.capacity_share(2.0, 65536, 128, 2) == 2048
    assert oracle.capacity_share(1.0, 100, 8, 2) == 25


# ----------------------------------------------------------------------------- generator
def test_workload_generator_statistics_and_determinism():
    w = wl.CONFIGS["tiny_f32"]
    a = wl.make_inputs(w)
    b = wl.make_inputs(w)
    for key in ("x", "wg", "w1", "w2"):
        assert torch.equal(a[key], b[key])
    assert abs(float(a["x"].std()) - 0.02) < 5e-4
    assert abs(float(a["wg"].std()) - 1 / np.sqrt(w.D)) < 2e-3
    assert abs(float(a["w1"].mean())) < 1e-4
    # slices can be drawn independently
    row = wl.normal(w.seed, wl.STREAM_X, (w.D,), 0.02, torch.float32, start=5 * w.D)
    assert torch.equal(row, a["x"][5])
    lm = wl.CONFIGS["lm"]
    bias = wl.zipf_bias(lm)
    assert bias.shape == (64,) and float(bias.max()) == 0.0
    assert float(bias.min()) == pytest.approx(-0.8 * 0.25 * 0.02 * np.log(64), rel=1e-5)


def test_skewed_workload_has_a_hot_expert(oracle):
    """The skewed workload's gate offsets must give a hot expert above 10 % of the
    assignments and leave no expert idle (checked on a token subsample)."""
    w = wl.CONFIGS["skewed_large"].scaled(T=8192)
    x = wl.normal(w.seed, wl.STREAM_X, (w.T, w.D), 0.02, torch.bfloat16)
    wg = wl.normal(w.seed, wl.STREAM_WG, (w.E, w.D), 1 / np.sqrt(w.D), torch.bfloat16)
    logits = oracle.gate_logits(x, wg, wl.zipf_bias(w))
    idx, _ = oracle.topk(logits, 2)
    counts, *_ = oracle.route(idx, w.E)
    share = counts / counts.sum()
    assert share.max() > 0.10
    assert (counts > 0).sum() >= 120
