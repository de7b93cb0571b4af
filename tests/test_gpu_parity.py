"""GPU parity: every C-ABI entry point of the dynamic-gating path against the CPU oracle,
element by element on the same seeded inputs.

Bars: bit-exact for indices, counts, offsets and the permutation; layer output within
2e-2 (bf16) / 1e-5 (fp32) normalised max error against the fp64 oracle.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from paper_2303_06182_amd import binding, workloads as wl
from helpers import (LOGIT_ATOL, LOGIT_RTOL, RMS_TOL, TOL, W_TOL, guarded_inputs, norm_max_err, p999_rel_err,
                     rms_rel_err, to_np, worst_row_rms_rel_err)

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load_library()
    return torch.device("cuda:0")


def layer_for(w: wl.Workload, renormalize=True, T_max=None):
    return binding.MoeLayer(T_max if T_max is not None else w.T, w.D, w.F, w.E, w.k, w.dtype, renormalize)


def cuda(inp):
    return {k: (None if v is None else v.cuda()) for k, v in inp.items()}


def check_logits(got, ref):
    tol = LOGIT_RTOL * np.abs(ref).max() + LOGIT_ATOL
    assert np.abs(got.astype(np.float64) - ref.astype(np.float64)).max() <= tol


# ----------------------------------------------------------------------------- gate + top-k
def test_topk_on_hand_made_logits_with_exact_ties(dev):
    """fp32 gate with an identity gate matrix reproduces x as logits exactly, so hand-made
    logits (ties included) reach the top-k kernel unchanged."""
    E, D = 12, 16
    l = np.zeros((6, D), dtype=np.float32)
    l[1, 5] = l[1, 9] = 2.0                  # duplicated maximum: 5 before 9
    l[2, 11] = 1.0
    l[2, 0] = l[2, 7] = 0.5                  # tie for second place: 0
    l[3, :E] = np.linspace(-1, 1, E)
    l[4, :E] = -3.0                          # all equal (negative)
    l[5, :E] = np.array([1, 1, 1, 0, 0, 0, 1, 1, 1, 0, 0, 0], dtype=np.float32)
    wg = np.zeros((E, D), dtype=np.float32)
    wg[np.arange(E), np.arange(E)] = 1.0
    for k in (1, 2, 3):
        m = binding.MoeLayer(8, D, 64, E, k, "f32")
        logits, idx, w = m.moe_gate_topk(torch.from_numpy(l).cuda(), torch.from_numpy(wg).cuda())
        np.testing.assert_array_equal(to_np(logits), l[:, :E])
        ridx, rw = orc.topk(l[:, :E], k)
        np.testing.assert_array_equal(to_np(idx), ridx)
        np.testing.assert_allclose(to_np(w), rw, rtol=W_TOL)
    if k >= 2:
        np.testing.assert_array_equal(to_np(idx)[:3, :2], [[0, 1], [5, 9], [11, 0]])


GATE_CASES = [
    # name, dtype, T, D, E, k, renorm, zipf, gate_scale
    ("f32_e8", "f32", 300, 64, 8, 2, True, 0.0, 1.0),
    ("f32_e5_k3_sharp", "f32", 130, 40, 5, 3, False, 0.0, 100.0),
    # K a multiple of 32: the fp32 MFMA kernel; E = 5 / 70 / 12 take its scalar, ragged and 16-byte stores
    ("f32_mfma_e5", "f32", 130, 64, 5, 3, False, 0.0, 100.0),
    ("f32_mfma_e70", "f32", 333, 96, 70, 2, True, 0.0, 50.0),
    ("f32_mfma_e12_long", "f32", 65, 1024, 12, 2, True, 0.0, 30.0),
    ("bf16_e64_zipf", "bf16", 1000, 256, 64, 2, True, 0.8, 1.0),
    ("bf16_e128_sharp", "bf16", 777, 512, 128, 2, True, 1.2, 100.0),
    ("bf16_e200_k4", "bf16", 200, 128, 200, 4, False, 0.0, 50.0),
    ("bf16_e16_k1", "bf16", 513, 72, 16, 1, True, 0.0, 30.0),
    ("bf16_e1000_k8", "bf16", 70, 64, 1000, 8, True, 0.0, 100.0),
    ("bf16_e3_k3", "bf16", 64, 64, 3, 3, True, 0.0, 100.0),
    # few tokens, long K: the gate GEMM is cut along K into slices that the top-k kernel adds up
    ("bf16_splitk_e128", "bf16", 100, 1024, 128, 2, True, 0.0, 30.0),
    ("bf16_splitk_e37", "bf16", 33, 2048, 37, 3, False, 0.0, 30.0),
    ("bf16_splitk_t1", "bf16", 1, 4096, 16, 2, True, 0.0, 30.0),
    # more than 256 tokens, bf16, E <= 128, D a multiple of 64: the gate GEMM decides the routing in its epilogue.
    # Tile heights 32 / 64 / 128 / 256 rows (by T), 1 to 4 column blocks (by E), E not a multiple of 4 or 32,
    # k = 1 .. 8, raw softmax, a ragged last tile
    ("bf16_fused_e37_k3", "bf16", 3001, 192, 37, 3, False, 0.0, 40.0),
    ("bf16_fused_e8_k8", "bf16", 600, 64, 8, 8, True, 0.0, 40.0),
    ("bf16_fused_e96_t33k", "bf16", 33000, 128, 96, 2, True, 1.0, 40.0),
    ("bf16_fused_e8_t70k", "bf16", 70001, 64, 8, 1, True, 0.0, 40.0),
    ("bf16_fused_e64_t66k_k4", "bf16", 66000, 64, 64, 4, False, 0.8, 40.0),
    ("bf16_fused_e128_t17k", "bf16", 17000, 256, 128, 2, True, 1.2, 40.0),
    ("bf16_fused_e100_k5", "bf16", 9000, 128, 100, 5, True, 0.0, 40.0),
]


@pytest.mark.parametrize("case", GATE_CASES, ids=[c[0] for c in GATE_CASES])
def test_gate_topk_parity(dev, case):
    name, dtype, T, D, E, k, renorm, zipf, gs = case
    w = wl.Workload(name, dtype, T=T, D=D, F=64, E=E, k=k, zipf_s=zipf, zipf_c=0.5, gate_scale=gs, seed=77)
    say("gate case", case)
    inp, redraws = guarded_inputs(w)
    g = cuda(inp)
    m = layer_for(w, renorm)
    logits, idx, gw = m.moe_gate_topk(g["x"], g["wg"], g["gate_bias"])
    torch.cuda.synchronize()
    ref_logits = orc.gate_logits(inp["x"], inp["wg"], inp["gate_bias"])
    check_logits(to_np(logits), ref_logits)
    # stage exactness: the oracle's top-k of the GPU's own logits
    sidx, sw = orc.topk(to_np(logits), k, renorm)
    np.testing.assert_array_equal(to_np(idx), sidx)
    np.testing.assert_allclose(to_np(gw), sw, rtol=W_TOL, atol=1e-30)
    # end to end: with the margin guard the decision equals the oracle's
    ridx, rw = orc.topk(ref_logits, k, renorm)
    np.testing.assert_array_equal(to_np(idx), ridx)
    np.testing.assert_allclose(to_np(gw), rw, rtol=1e-4)


@pytest.mark.parametrize("T,D,E,k", [(3000, 256, 128, 2), (700, 128, 37, 3), (40, 512, 64, 2), (500, 72, 16, 2)])
def test_gate_topk_without_logits_output(dev, T, D, E, k):
    """logits_out = NULL with a workspace: the decision must not depend on whether the logits are written out
    (large bf16 batches keep them in registers, the other paths park them in the workspace), and the whole layer
    must give the same y whether or not any routing array is requested."""
    w = wl.Workload("nologits", "bf16", T=T, D=D, F=128, E=E, k=k, zipf_s=0.8, zipf_c=0.5, gate_scale=30.0, seed=5)
    g = cuda(wl.make_inputs(w))
    m = layer_for(w)
    logits, idx, gw = m.moe_gate_topk(g["x"], g["wg"], g["gate_bias"])
    idx2 = torch.full_like(idx, -1)
    gw2 = torch.full_like(gw, float("nan"))
    ws, wsb = m._ws()
    rc = m.lib.moe_gate_topk(m.h, binding._ptr(g["x"]), binding._ptr(g["wg"]), binding._ptr(g["gate_bias"]), T, None,
                             binding._ptr(idx2), binding._ptr(gw2), ws, wsb, binding._stream())
    assert rc == binding.MOE_OK
    # neither logits nor workspace: an argument error, nothing launched
    rc = m.lib.moe_gate_topk(m.h, binding._ptr(g["x"]), binding._ptr(g["wg"]), None, T, None, binding._ptr(idx2),
                             binding._ptr(gw2), None, 0, binding._stream())
    assert rc == binding.MOE_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(gw, gw2)
    y_all = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"], routing_out=m.empty_routing(T))
    y_none = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"])
    y_counts = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"],
                                   routing_out=dict(counts=torch.empty(E, dtype=torch.int32, device="cuda")))
    torch.cuda.synchronize()
    assert torch.equal(y_all, y_none) and torch.equal(y_all, y_counts)


# ----------------------------------------------------------------------------- routing
def random_idx(T, E, k, seed, skew=False):
    rng = np.random.default_rng(seed)
    if skew:
        p = 1.0 / np.arange(1, E + 1) ** 1.5
        p /= p.sum()
    else:
        p = np.full(E, 1.0 / E)
    out = np.empty((T, k), dtype=np.int32)
    for t in range(T):
        out[t] = rng.choice(E, size=k, replace=False, p=p)
    return out


ROUTE_CASES = [(1, 4, 2, False), (64, 128, 2, False), (255, 8, 2, False), (256, 8, 2, True), (257, 16, 1, False),
               (1000, 128, 2, True), (5000, 64, 2, True), (777, 1000, 8, False), (4096, 3, 3, False),
               (3000, 1, 1, False), (20000, 128, 2, True),
               # around the limit of the single-block kernel for small batches (4096 assignments)
               (2048, 16, 2, True), (2049, 16, 2, False), (512, 1000, 8, False), (130, 1024, 8, False)]


@pytest.mark.parametrize("T,E,k,skew", ROUTE_CASES)
def test_route_counts_bit_exact(dev, T, E, k, skew):
    say("route case", T, E, k, skew)
    idx = random_idx(T, E, k, seed=T + E, skew=skew)
    m = binding.MoeLayer(T, 64, 64, E, k, "bf16")
    counts, offsets, dst_row, src_tok = m.moe_route_counts(torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    rc, ro, rd, rs = orc.route(idx, E)
    np.testing.assert_array_equal(to_np(counts), rc)
    np.testing.assert_array_equal(to_np(offsets), ro)
    np.testing.assert_array_equal(to_np(dst_row), rd)
    np.testing.assert_array_equal(to_np(src_tok), rs)


@pytest.mark.parametrize("T", [700, 5000])   # below and above the single-block kernel's 4096 assignments
def test_route_with_a_repeated_expert_inside_a_token(dev, T):
    """The k experts of a token are distinct by construction (top-k selection, Sec. 2.3); handed a token that
    names one expert twice, the routing still has to be a permutation -- both kernels rank such assignments
    in (token, slot) order -- and everything around it must equal the oracle."""
    E, k = 16, 2
    idx = random_idx(T, E, k, seed=T, skew=True)
    dup = [3, T // 2, T - 1]
    idx[dup, 1] = idx[dup, 0]
    m = binding.MoeLayer(T, 64, 64, E, k, "bf16")
    counts, offsets, dst_row, src_tok = [to_np(a) for a in m.moe_route_counts(torch.from_numpy(idx).cuda())]
    torch.cuda.synchronize()
    np.testing.assert_array_equal(counts, np.bincount(idx.ravel(), minlength=E))
    np.testing.assert_array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    assert sorted(dst_row.ravel().tolist()) == list(range(T * k))           # a bijection onto the rows
    for t in range(T):
        for j in range(k):
            r = dst_row[t, j]
            assert offsets[idx[t, j]] <= r < offsets[idx[t, j] + 1] and src_tok[r] == t
    for t in dup:
        assert dst_row[t, 1] == dst_row[t, 0] + 1                          # slot order inside the token
    for e in range(E):                                                     # ascending tokens inside an expert
        rows = src_tok[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(rows) >= 0)


def test_route_all_tokens_to_one_expert_and_T_zero(dev):
    T, E, k = 1500, 32, 2
    idx = np.empty((T, k), dtype=np.int32)
    idx[:, 0] = 7
    idx[:, 1] = 30
    m = binding.MoeLayer(T, 64, 64, E, k, "bf16")
    out = m.moe_route_counts(torch.from_numpy(idx).cuda())
    ref = orc.route(idx, E)
    for a, b in zip(out, ref):
        np.testing.assert_array_equal(to_np(a), b)
    out0 = m.moe_route_counts(torch.empty((0, k), dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert int(out0[0].sum()) == 0 and int(out0[1].abs().sum()) == 0


# ----------------------------------------------------------------------------- dispatch / combine
@pytest.mark.parametrize("dtype,T,D,E,k", [("bf16", 1000, 1024, 64, 2), ("bf16", 333, 72, 8, 3), ("f32", 257, 512, 8, 2),
                                           ("bf16", 1, 2048, 128, 2), ("f32", 50, 8, 4, 1)])
def test_dispatch_and_combine(dev, dtype, T, D, E, k):
    say("dispatch/combine case", dtype, T, D, E, k)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = wl.normal(5, 0, (T, D), 1.0, tdt)
    idx = random_idx(T, E, k, seed=9, skew=True)
    rc, ro, rd, rs = orc.route(idx, E)
    m = binding.MoeLayer(T, D, 64, E, k, dtype)
    d_dst = torch.from_numpy(rd).cuda()
    xp = m.moe_dispatch(x.cuda(), d_dst)
    torch.cuda.synchronize()
    ref_xp = orc.dispatch(x, rs)
    np.testing.assert_array_equal(to_np(xp).astype(np.float64), ref_xp)      # a copy: bit exact
    # combine on fresh rows
    yp = wl.normal(6, 1, (T * k, D), 1.0, tdt)
    gw = np.random.default_rng(3).random((T, k)).astype(np.float32)
    y = m.moe_combine(yp.cuda(), d_dst, torch.from_numpy(gw).cuda())
    torch.cuda.synchronize()
    ref_y = orc.combine(to_np(yp), rd, gw)
    err = norm_max_err(to_np(y), ref_y)
    assert err <= (4e-3 if dtype == "bf16" else 2e-7), err     # one rounding of the output


# ----------------------------------------------------------------------------- grouped expert FFN
FFN_CASES = [
    # dtype, counts per expert (ragged, with empty experts), D, F, bias
    ("bf16", [130, 0, 257, 1, 64, 0, 33, 515], 256, 512, False),
    ("bf16", [5, 0, 0, 1, 2, 0, 3, 0, 0, 1, 1, 0], 128, 192, True),
    ("bf16", [700, 45], 72, 136, True),
    ("bf16", [64] * 16, 512, 1024, False),
    ("f32", [100, 0, 37, 64, 1], 64, 128, True),
    ("f32", [300], 128, 256, False),
    # fp32: D a multiple of 32 but F not (first GEMM on the MFMA kernel, second on the vector-FMA kernel),
    # and the other way round; many K tiles, several M tiles per expert with ragged ends
    ("f32", [65, 0, 130, 1], 96, 72, True),
    ("f32", [65, 0, 130, 1], 72, 96, True),
    ("f32", [200, 63, 64, 0, 129], 1024, 160, False),
    # 256-row tiles: 24 M tiles x 13 N tiles = 312 tiles on 256 CUs -> one whole round in the main
    # launch, 56 leftover tiles as 128x128 sub-tiles in the tail launch; the second GEMM (24 tiles)
    # runs in the tail launch alone
    ("bf16", [1100, 0, 900, 257, 1500, 640, 3, 700], 256, 3328, False),
    # 24 x 17 = 408 tiles: the 152 leftover tiles are too many for the tail launch, two main rounds
    ("bf16", [1100, 0, 900, 257, 1500, 640, 3, 700], 256, 4352, True),
    # 256-row tiles whose last column tile is partly outside the matrix, in both GEMMs (F = 12.5, D = 11.25 column
    # tiles; 24 x 13 and 24 x 12 tiles: a whole round each in the main launch), with offsets
    ("bf16", [1100, 0, 900, 257, 1500, 640, 3, 700], 2880, 3200, True),
    # a single K tile per output tile in the first GEMM (the load stream changes tile after every K tile)
    ("bf16", [1100, 0, 900, 257, 1500, 640, 3, 700], 64, 3328, False),
]


@pytest.mark.parametrize("case", FFN_CASES, ids=[str(i) for i in range(len(FFN_CASES))])
def test_expert_ffn_parity(dev, case):
    dtype, counts, D, F, bias = case
    say("ffn case", case)
    E = len(counts)
    N = int(sum(counts))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    xp = wl.normal(11, 0, (N, D), 1.0, tdt)
    w1 = wl.normal(11, 1, (E, F, D), 1.0 / np.sqrt(D), tdt)
    w2 = wl.normal(11, 2, (E, D, F), 1.0 / np.sqrt(F), tdt)
    b1 = wl.normal(11, 3, (E, F), 0.5, tdt) if bias else None
    b2 = wl.normal(11, 4, (E, D), 0.5, tdt) if bias else None
    # idle experts are poisoned: their weights must never be read into a result
    w1g, w2g = w1.clone(), w2.clone()
    for e, c in enumerate(counts):
        if c == 0:
            w1g[e] = float("nan")
            w2g[e] = float("nan")
    m = binding.MoeLayer(N, D, F, E, 1, dtype)      # k = 1: T_max * k = N rows
    yp = m.moe_expert_ffn(xp.cuda(), torch.from_numpy(offsets).cuda(), w1g.cuda(), w2g.cuda(),
                          None if b1 is None else b1.cuda(), None if b2 is None else b2.cuda())
    torch.cuda.synchronize()
    ref = orc.expert_ffn(xp, offsets, w1, w2, b1, b2)
    got = to_np(yp)
    assert np.all(np.isfinite(got))
    err = norm_max_err(got, ref)
    rms = rms_rel_err(got, ref)
    say("  ffn err", err, "rms", rms, "worst row rms", worst_row_rms_rel_err(got, ref))
    assert err <= TOL[dtype], err
    assert rms <= RMS_TOL[dtype], rms


# ----------------------------------------------------------------------------- the whole layer
def routing_sample(w, n, counts, offsets, src_tok, tile=256):
    """Token sample for a full-size comparison, built from the routing so that no region of the expert GEMMs'
    row space goes unchecked: for every expert with rows its first row, its last row, the first row of its last
    (ragged) M tile and a row in the middle of that tile; the last 2 * tile rows of the whole row space and a
    stride through its last eighth (the tiles of the last, partly filled round of a persistent launch are cut out
    of the end of the tile list and run by a second launch with a smaller tile shape); then a seeded random fill
    up to n tokens."""
    N = int(offsets[-1])
    rows = []
    for e in range(w.E):
        c = int(counts[e])
        if c == 0:
            continue
        a, b = int(offsets[e]), int(offsets[e + 1])
        last_tile = a + ((c - 1) // tile) * tile
        rows += [a, b - 1, last_tile, (last_tile + b - 1) // 2]
    rows += list(range(max(0, N - 2 * tile), N))
    rows += list(range(N - N // 8, N, 97))
    tokens = np.unique(src_tok[np.array(rows, dtype=np.int64)])
    if tokens.size < n:
        rest = np.random.default_rng(w.seed).permutation(w.T)
        rest = rest[~np.isin(rest, tokens)][:n - tokens.size]
        tokens = np.union1d(tokens, rest)
    return tokens.astype(np.int32)


def run_layer_and_check(w: wl.Workload, sample=None, with_ffn_bias=False, renorm=True, device="cpu"):
    inp, redraws = guarded_inputs(w, device=device, with_ffn_bias=with_ffn_bias)
    g = cuda(inp)
    host = {k: (None if v is None else v.cpu()) for k, v in inp.items()}
    m = layer_for(w, renorm)
    r = m.empty_routing(w.T)
    y = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"], g["b1"], g["b2"], routing_out=r)
    torch.cuda.synchronize()
    ref_logits = orc.gate_logits(host["x"], host["wg"], host["gate_bias"])
    check_logits(to_np(r["logits"]), ref_logits)
    ridx, rw = orc.topk(ref_logits, w.k, renorm)
    np.testing.assert_array_equal(to_np(r["topk_idx"]), ridx)                 # bit-exact routing
    np.testing.assert_allclose(to_np(r["topk_w"]), rw, rtol=1e-4)
    rc, ro, rd, rs = orc.route(ridx, w.E)
    np.testing.assert_array_equal(to_np(r["counts"]), rc)
    np.testing.assert_array_equal(to_np(r["offsets"]), ro)
    np.testing.assert_array_equal(to_np(r["dst_row"]), rd)
    np.testing.assert_array_equal(to_np(r["src_tok"]), rs)
    assert int(rc.sum()) == w.k * w.T
    if sample is None or sample >= w.T:
        tokens = None
    else:
        tokens = routing_sample(w, sample, rc, ro, rs)
    ref_y = orc.layer_tokens(host["x"], host["w1"], host["w2"], ridx, rw, tokens=tokens, b1=host["b1"], b2=host["b2"])
    got = to_np(y)
    assert np.all(np.isfinite(got))
    got_rows = got if tokens is None else got[tokens]
    err = norm_max_err(got_rows, ref_y)
    rms = rms_rel_err(got_rows, ref_y)
    row = worst_row_rms_rel_err(got_rows, ref_y)
    say("  %s: T=%d compared=%d redraws=%d max share=%.3f idle experts=%d  err=%.3e rms=%.3e worst row rms=%.3e  "
        "99.9th pct rel err=%.3e" %
        (w.name, w.T, got_rows.shape[0], redraws, rc.max() / rc.sum(), int((rc == 0).sum()), err, rms, row,
         p999_rel_err(got_rows, ref_y)))
    assert err <= TOL[w.dtype], err
    assert rms <= RMS_TOL[w.dtype], rms
    assert row <= 4 * RMS_TOL[w.dtype], row     # no single token row off by more than rounding either
    return dict(err=err, counts=rc, y=y, routing=r)


SMALL = [
    wl.CONFIGS["tiny_f32"].scaled(T=200, D=128, F=256),
    wl.CONFIGS["tiny_f32"].scaled(name="tiny_f32_sharp", T=130, D=64, F=128, gate_scale=100.0),
    wl.CONFIGS["lm"].scaled(T=1000, D=256, F=512),
    wl.CONFIGS["lm"].scaled(name="lm_sharp", T=777, D=256, F=512, gate_scale=100.0),
    wl.CONFIGS["mt_encoder"].scaled(T=2500, D=256, F=512),
    wl.CONFIGS["mt_decoder"].scaled(D=256, F=512),
    wl.CONFIGS["skewed_large"].scaled(T=3000, D=128, F=256),
    wl.CONFIGS["lm"].scaled(name="lm_k1", T=500, D=128, F=256, k=1, gate_scale=100.0),
    wl.CONFIGS["lm"].scaled(name="e4_k4", T=300, D=128, F=256, E=4, k=4, gate_scale=100.0, zipf_s=0.0),
    wl.CONFIGS["lm"].scaled(name="e1_k1", T=300, D=128, F=256, E=1, k=1, zipf_s=0.0),
    wl.CONFIGS["lm"].scaled(name="odd_dims", T=301, D=72, F=136, E=6, k=2, gate_scale=100.0),
    # the limits of the configuration space: E = MOE_MAX_E, k = MOE_MAX_K, E not a multiple of 4
    wl.CONFIGS["lm"].scaled(name="e1024_k8", T=260, D=64, F=64, E=1024, k=8, gate_scale=100.0, zipf_s=0.0),
    wl.CONFIGS["lm"].scaled(name="e1024_k1_f32", dtype="f32", T=70, D=64, F=64, E=1024, k=1, gate_scale=100.0,
                            zipf_s=0.0),
    wl.CONFIGS["lm"].scaled(name="e37_k3", T=513, D=192, F=320, E=37, k=3, gate_scale=100.0),
    wl.CONFIGS["lm"].scaled(name="e130_k2", T=257, D=128, F=128, E=130, k=2, gate_scale=100.0, zipf_s=0.0),
]


@pytest.mark.parametrize("w", SMALL, ids=[w.name for w in SMALL])
def test_layer_forward_small(dev, w):
    say("layer small", w)
    run_layer_and_check(w)


def test_layer_forward_with_biases_and_raw_softmax(dev):
    w = wl.CONFIGS["lm"].scaled(name="lm_bias", T=600, D=128, F=256, gate_scale=100.0)
    run_layer_and_check(w, with_ffn_bias=True, renorm=False)
    w = wl.CONFIGS["tiny_f32"].scaled(name="f32_bias", T=150, D=64, F=128, gate_scale=100.0)
    run_layer_and_check(w, with_ffn_bias=True, renorm=False)


# every token of the first four workloads (the oracle needs 1 s for lm, about 10 s for mt_encoder on the box's
# cores); skewed_large on 8192 tokens chosen from the routing (routing_sample)
FULL = [("tiny_f32", None), ("lm", None), ("mt_encoder", None), ("mt_decoder", None), ("skewed_large", 8192)]


def test_layer_forward_large_tiles_with_odd_dimensions(dev):
    """A mid-size layer on the 256-row tiles' main launch (8 experts with about 5000 rows each: 160 row tiles x 13
    and x 2 column tiles) whose dimensions are not multiples of the tile: D = 320 (five K tiles, a column tile and
    a quarter in the second GEMM), F = 3200 (12.5 column tiles in the first GEMM, 50 K tiles in the second), with
    offsets in both GEMMs and the rows of the first gathered from x; every token compared."""
    w = wl.CONFIGS["mt_encoder"].scaled(name="ring_odd", T=20000, D=320, F=3200, E=8)
    say("layer large tiles, odd dimensions", w)
    run_layer_and_check(w, with_ffn_bias=True, device="cuda")


@pytest.mark.parametrize("name,sample", FULL, ids=[f[0] for f in FULL])
def test_layer_forward_full_size(dev, name, sample):
    """The five benchmark workloads at full size: routing bit-exact for every token; output compared on every
    token, for skewed_large on a sample of 8192 tokens that the oracle computes one by one (each output row
    depends only on its own token, so a sample is exact) and that covers every expert's first, last and
    ragged-tile rows and the end of the row space."""
    w = wl.CONFIGS[name]
    say("layer full size", w)
    out = run_layer_and_check(w, sample=sample, device="cuda")
    rc = out["counts"]
    if name == "skewed_large":
        assert rc.max() / rc.sum() > 0.10          # a hot expert above 10 % of the assignments
    if name == "mt_decoder":
        assert rc.max() <= 8 and (rc == 0).sum() > 20
    del out
    torch.cuda.empty_cache()


def test_idle_experts_weights_never_read(dev):
    w = wl.CONFIGS["lm"].scaled(name="idle", T=400, D=128, F=256, E=8, zipf_s=0.0, gate_scale=100.0)
    inp, _ = guarded_inputs(w)
    bias = torch.zeros(w.E)
    bias[[2, 5]] = -1e4                     # experts 2 and 5 never win
    inp["gate_bias"] = bias
    g = cuda(inp)
    m = layer_for(w)
    r = m.empty_routing(w.T)
    y0 = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"], routing_out=r).clone()
    assert int(r["counts"][2]) == 0 and int(r["counts"][5]) == 0
    g["w1"][[2, 5]] = float("nan")
    g["w2"][[2, 5]] = float("nan")
    y1 = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"])
    torch.cuda.synchronize()
    assert torch.isfinite(y1.float()).all()
    assert torch.equal(y0, y1)


def test_T_zero_T_one_and_T_below_T_max(dev):
    w = wl.CONFIGS["lm"].scaled(name="edge", T=1, D=128, F=256, E=8, zipf_s=0.0, gate_scale=100.0)
    run_layer_and_check(w)
    inp = cuda(wl.make_inputs(w))
    m = binding.MoeLayer(512, w.D, w.F, w.E, w.k, w.dtype)
    y = m.moe_layer_forward(inp["x"][:0], inp["wg"], inp["w1"], inp["w2"])
    torch.cuda.synchronize()
    assert y.shape == (0, w.D)
    # a handle made for T_max serves any smaller T
    w2 = w.scaled(T=300)
    inp2, _ = guarded_inputs(w2)
    g2 = cuda(inp2)
    ya = m.moe_layer_forward(g2["x"], g2["wg"], g2["w1"], g2["w2"])
    yb = layer_for(w2).moe_layer_forward(g2["x"], g2["wg"], g2["w1"], g2["w2"])
    torch.cuda.synchronize()
    assert torch.equal(ya, yb)


def test_layer_forward_is_deterministic(dev):
    w = wl.CONFIGS["skewed_large"].scaled(T=5000, D=256, F=512)
    g = cuda(wl.make_inputs(w))
    m = layer_for(w)
    outs = []
    for _ in range(3):
        r = m.empty_routing(w.T)
        y = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"], routing_out=r)
        torch.cuda.synchronize()
        outs.append((y.clone(), r["dst_row"].clone(), r["src_tok"].clone(), r["topk_w"].clone()))
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert torch.equal(a, b)


def test_stagewise_calls_equal_the_fused_call(dev):
    w = wl.CONFIGS["lm"].scaled(T=900, D=256, F=512)
    g = cuda(wl.make_inputs(w))
    m = layer_for(w)
    r = m.empty_routing(w.T)
    y = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"], routing_out=r)
    logits, idx, gw = m.moe_gate_topk(g["x"], g["wg"], g["gate_bias"])
    counts, offsets, dst_row, src_tok = m.moe_route_counts(idx)
    xp = m.moe_dispatch(g["x"], dst_row)
    yp = m.moe_expert_ffn(xp, offsets, g["w1"], g["w2"])
    y2 = m.moe_combine(yp, dst_row, gw)
    torch.cuda.synchronize()
    assert torch.equal(idx, r["topk_idx"]) and torch.equal(dst_row, r["dst_row"]) and torch.equal(counts, r["counts"])
    assert torch.equal(y, y2)


# ----------------------------------------------------------------------------- error paths (host side)
def test_argument_errors(dev):
    w = wl.CONFIGS["lm"].scaled(T=64, D=128, F=256, E=8, zipf_s=0.0)
    g = cuda(wl.make_inputs(w))
    m = layer_for(w)
    with pytest.raises(binding.MoeError) as e:
        m.moe_layer_forward(torch.cat([g["x"], g["x"]]), g["wg"], g["w1"], g["w2"])      # T > T_max
    assert e.value.code == binding.MOE_ERR_INVALID_ARG
    with pytest.raises(binding.MoeError) as e:
        m.moe_dispatch(g["x"].view(-1)[1:1 + (w.T - 1) * w.D].view(w.T - 1, w.D),
                       torch.zeros((w.T - 1, 2), dtype=torch.int32, device="cuda"))       # misaligned x
    assert e.value.code == binding.MOE_ERR_INVALID_ARG
    small = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, w.dtype, alloc_workspace=False)
    small.workspace = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.MoeError) as e:
        small.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"])
    assert e.value.code == binding.MOE_ERR_WORKSPACE
    torch.cuda.synchronize()


@pytest.mark.parametrize("kind", ["bf16_mid", "bf16_large_tiles", "bf16_decoder", "w8_decoder", "w4_decoder"])
def test_layer_forward_can_be_captured_in_a_graph(dev, kind):
    """The fused call only enqueues kernels on the caller's stream (no allocation, no host wait,
    no memset node), so it can be recorded into a HIP graph; every replay, with eager work and
    synchronisations in between, must reproduce the eager result bit for bit.  The decoder-sized
    cases take the small-batch kernels (gate GEMM split along K, single-block routing) and the
    quantised expert GEMMs through the same check."""
    if kind == "bf16_mid":
        w = wl.CONFIGS["lm"].scaled(name="graph", T=1500, D=256, F=512, E=16)
    elif kind == "bf16_large_tiles":
        # 256-row tiles: main launch (the ring-of-K-steps kernel, all of the CU's LDS) and tail launch in the graph
        w = wl.CONFIGS["mt_encoder"].scaled(name="graph_large", T=6000, D=256, F=3328, E=8)
    else:
        w = wl.CONFIGS["mt_decoder"].scaled(name="graph_dec", D=512, F=1024, E=32)
    g = cuda(wl.make_inputs(w))
    m = layer_for(w)
    y_eager = torch.empty((w.T, w.D), dtype=torch.bfloat16, device="cuda")
    y_graph = torch.empty_like(y_eager)
    if kind == "w8_decoder":
        q1, s1 = m.moe_quantize_e4m3(g["w1"])
        q2, s2 = m.moe_quantize_e4m3(g["w2"])
    elif kind == "w4_decoder":
        q1, s1 = m.moe_quantize_mxfp4(g["w1"])
        q2, s2 = m.moe_quantize_mxfp4(g["w2"])

    def step(out):
        if kind == "w8_decoder":
            m.moe_layer_forward_w8(g["x"], g["wg"], q1, q2, s1, s2, g["gate_bias"], y=out)
        elif kind == "w4_decoder":
            m.moe_layer_forward_w4(g["x"], g["wg"], q1, q2, s1, s2, g["gate_bias"], y=out)
        else:
            m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"], y=out)

    for _ in range(3):
        step(y_eager)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(y_graph)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(y_graph)
    for _ in range(4):
        y_graph.zero_()
        graph.replay()
        step(y_eager)
        torch.cuda.synchronize()
        assert torch.equal(y_eager, y_graph)
