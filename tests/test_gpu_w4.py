"""GPU parity of the weight-only 4-bit (e2m1 + e8m0 block scales) expert-weight path, through the
C-ABI: the quantiser nibble for nibble and scale byte for scale byte against the CPU oracle, and the
expert FFN / the whole layer against the fp64 oracle fed the dequantised weights (scale * value is
exactly a bf16 number, so both sides see identical operands and the bar is the bf16 path's)."""
import sys

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from oracle import quant_mxfp4 as oq
from paper_2303_06182_amd import binding, workloads as wl
from helpers import TOL, guarded_inputs, norm_max_err, to_np

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load_library()
    return torch.device("cuda:0")


def dequant_bf16(codes: np.ndarray, sb: np.ndarray) -> torch.Tensor:
    d = oq.dequantize(codes, sb)
    t = torch.from_numpy(d.astype(np.float32)).to(torch.bfloat16)
    assert np.array_equal(t.float().numpy().astype(np.float64), d), "scale * value must be exact in bf16"
    return t


def same_codes(got, ref):
    """Equal nibbles, except that +0 and -0 are one number."""
    return (got == ref) | (((got | ref) & 0x7) == 0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_quantizer_nibbles_and_scales_equal_the_oracle(dev, dtype):
    say("mxfp4 quantizer", dtype)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    E, rows, cols = 5, 96, 640            # cols not a multiple of 512: a padded scale group
    w = wl.normal(41, 0, (E, rows, cols), 1.0, tdt)
    mul = torch.tensor([1e-3, 0.02, 1.0, 30.0, 1.0]).reshape(E, 1, 1)
    w = (w.float() * mul).to(tdt)
    w[4, 0, :32] = 0.0                    # an all-zero block
    w[4, 1, :32] = 0.0
    w[4, 1, 5] = 6.0                      # block maximum exactly 6 * 2^0: the scale must not grow
    w[4, 2, :32] = 0.0
    w[4, 2, 7] = -3.0                     # exactly 6 * 2^-1
    # every tie of the grid at scale 1: the block's maximum 6 keeps the scale at 1
    w[4, 3, :32] = 0.0
    w[4, 3, 0] = 6.0
    ties = torch.tensor([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    w[4, 3, 1:8] = ties.to(tdt)
    w[4, 3, 8:15] = (-ties).to(tdt)
    m = binding.MoeLayer(8, 64, 64, E, 1, dtype)
    q, s = m.moe_quantize_mxfp4(w.cuda())
    torch.cuda.synchronize()
    rc, rs = oq.quantize(w.float().numpy().astype(np.float64))
    got_s = oq.unblocked_scales(to_np(s), rows, cols)
    np.testing.assert_array_equal(got_s, rs)
    got_c = oq.unblocked_data(to_np(q), rows, cols)
    ok = same_codes(got_c, rc)
    assert ok.all(), int((~ok).sum())
    assert list(got_c[4, 3, 1:8]) == [0, 2, 2, 4, 4, 6, 6]


W4_FFN_CASES = [
    # counts per expert (ragged, with empty experts), D, F, bias
    ([130, 0, 257, 1, 64, 0, 33, 515], 256, 512, False),
    ([5, 0, 0, 1, 2, 0, 3, 0, 0, 1, 1, 0], 128, 192, True),
    ([16] * 32, 512, 1024, True),                  # few rows per expert: 32-row tiles, two scale groups along K
    ([64, 48, 100, 47, 70, 90], 192, 320, False),   # 64-row tiles; N = 320 / 192 not multiples of the tile width
    ([700, 45], 64, 64, True),
    ([3, 2, 0, 1], 1088, 576, False),               # K = 1088 = 17 K tiles: three scale groups, the last one short
    # 1000 tiles of one or two K tiles each on ~768 resident blocks: blocks run two tiles, and a scale group is
    # shorter than the load pipeline is deep
    ([2] * 1000, 64, 128, False),
]


@pytest.mark.parametrize("case", W4_FFN_CASES, ids=[str(i) for i in range(len(W4_FFN_CASES))])
def test_expert_ffn_w4_parity(dev, case):
    counts, D, F, bias = case
    say("w4 ffn case", case)
    E, N = len(counts), int(sum(counts))
    tdt = torch.bfloat16
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    xp = wl.normal(51, 0, (N, D), 1.0, tdt)
    w1 = wl.normal(51, 1, (E, F, D), 1.0 / np.sqrt(D), tdt)
    w2 = wl.normal(51, 2, (E, D, F), 1.0 / np.sqrt(F), tdt)
    w1[0] *= 37.0
    w2[E - 1] *= 1.0 / 64
    b1 = wl.normal(51, 3, (E, F), 0.5, tdt) if bias else None
    b2 = wl.normal(51, 4, (E, D), 0.5, tdt) if bias else None
    m = binding.MoeLayer(N, D, F, E, 1, "bf16")
    q1, s1 = m.moe_quantize_mxfp4(w1.cuda())
    q2, s2 = m.moe_quantize_mxfp4(w2.cuda())
    # idle experts are poisoned: the largest scale and the largest element would show in any result
    for e, c in enumerate(counts):
        if c == 0:
            q1[e] = 0x77
            q2[e] = 0x77
            s1[e] = 254
            s2[e] = 254
    yp = m.moe_expert_ffn_w4(xp.cuda(), torch.from_numpy(offsets).cuda(), q1, q2, s1, s2,
                             None if b1 is None else b1.cuda(), None if b2 is None else b2.cuda())
    torch.cuda.synchronize()
    rc1, rs1 = oq.quantize(w1.float().numpy().astype(np.float64))
    rc2, rs2 = oq.quantize(w2.float().numpy().astype(np.float64))
    ref = orc.expert_ffn(xp, offsets, dequant_bf16(rc1, rs1), dequant_bf16(rc2, rs2), b1, b2)
    got = to_np(yp)
    assert np.all(np.isfinite(got))
    err = norm_max_err(got, ref)
    say("  w4 ffn err", err)
    assert err <= TOL["bf16"], err


W4_LAYER = [
    wl.CONFIGS["mt_decoder"].scaled(name="w4_dec", D=256, F=512),
    wl.CONFIGS["lm"].scaled(name="w4_lm", T=1000, D=256, F=512),
    wl.CONFIGS["lm"].scaled(name="w4_e37_k3", T=513, D=192, F=320, E=37, k=3, gate_scale=100.0),
]


def run_w4_layer(w, device="cpu", check_experts=None):
    inp, _ = guarded_inputs(w, device=device, with_ffn_bias=True)
    g = {k: (None if v is None else v.cuda()) for k, v in inp.items()}
    host = {k: (None if v is None else v.cpu()) for k, v in inp.items() if k not in ("w1", "w2")}
    m = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, "bf16")
    q1, s1 = m.moe_quantize_mxfp4(g["w1"])
    q2, s2 = m.moe_quantize_mxfp4(g["w2"])
    r = m.empty_routing(w.T)
    y = m.moe_layer_forward_w4(g["x"], g["wg"], q1, q2, s1, s2, g["gate_bias"], g["b1"], g["b2"], routing_out=r)
    torch.cuda.synchronize()
    logits = orc.gate_logits(host["x"], host["wg"], host["gate_bias"])
    ridx, rw = orc.topk(logits, w.k, True)
    np.testing.assert_array_equal(to_np(r["topk_idx"]), ridx)
    rc, ro, rd, rs = orc.route(ridx, w.E)
    np.testing.assert_array_equal(to_np(r["dst_row"]), rd)
    np.testing.assert_array_equal(to_np(r["offsets"]), ro)
    # Reference weights: the oracle's own quantisation of the experts in check_experts (all, by default),
    # which must equal the library's; for the others in use, the library's bytes (the quantiser has its
    # own test) dequantised by the oracle.  Idle experts stay zero: the oracle never reads them.
    active = [e for e in range(w.E) if rc[e] > 0]
    own = set(active if check_experts is None else [e for e in active if e in check_experts])
    d1 = torch.zeros((w.E, w.F, w.D), dtype=torch.bfloat16)
    d2 = torch.zeros((w.E, w.D, w.F), dtype=torch.bfloat16)
    for e in active:
        for wt, q, s, d in ((g["w1"], q1, s1, d1), (g["w2"], q2, s2, d2)):
            rows, cols = wt.shape[1], wt.shape[2]
            codes = oq.unblocked_data(to_np(q[e:e + 1]), rows, cols)
            sb = oq.unblocked_scales(to_np(s[e:e + 1]), rows, cols)
            if e in own:
                rcodes, rsb = oq.quantize(wt[e:e + 1].float().cpu().numpy().astype(np.float64))
                np.testing.assert_array_equal(sb, rsb)
                assert same_codes(codes, rcodes).all()
                codes, sb = rcodes, rsb
            d[e] = dequant_bf16(codes, sb)[0]
    ref = orc.layer_tokens(host["x"], d1, d2, ridx, rw, b1=host["b1"], b2=host["b2"])
    got = to_np(y)
    assert np.all(np.isfinite(got))
    err = norm_max_err(got, ref)
    say("  %s: active experts=%d err=%.3e" % (w.name, len(active), err))
    assert err <= TOL["bf16"], err
    return y, g, (q1, q2, s1, s2)


@pytest.mark.parametrize("w", W4_LAYER, ids=[w.name for w in W4_LAYER])
def test_layer_forward_w4_small(dev, w):
    say("w4 layer", w)
    run_w4_layer(w)


def test_layer_forward_w4_equals_stagewise_calls(dev):
    w = wl.CONFIGS["mt_decoder"].scaled(name="w4_stage", D=256, F=512)
    y, g, (q1, q2, s1, s2) = run_w4_layer(w)
    m = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, "bf16")
    _, idx, tw = m.moe_gate_topk(g["x"], g["wg"], g["gate_bias"])
    counts, offsets, dst_row, src_tok = m.moe_route_counts(idx)
    xp = m.moe_dispatch(g["x"], dst_row)
    yp = m.moe_expert_ffn_w4(xp, offsets, q1, q2, s1, s2, g["b1"], g["b2"])
    y2 = m.moe_combine(yp, dst_row, tw)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    y16 = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"], g["b1"], g["b2"])
    torch.cuda.synchronize()
    rel = norm_max_err(to_np(y), to_np(y16))
    say("  w4 vs bf16 weights: normalised max difference %.3e" % rel)
    assert rel < 0.5


def test_layer_forward_w4_full_size_decoder(dev):
    w = wl.CONFIGS["mt_decoder"]
    say("w4 full", w)
    run_w4_layer(w, device="cuda", check_experts={0, 1, 2, 64, 127})
    torch.cuda.empty_cache()


def test_layer_forward_w4_full_size_lm(dev):
    """The headline workload's shape (64 experts, about 256 rows each): the 64-row tiles of the quantised path."""
    w = wl.CONFIGS["lm"]
    say("w4 full lm", w)
    run_w4_layer(w, device="cuda", check_experts={0, 31, 63})
    torch.cuda.empty_cache()


def test_w4_argument_errors(dev):
    m = binding.MoeLayer(64, 72, 128, 4, 2, "bf16")      # D not a multiple of 64
    x = torch.zeros(8, 72, dtype=torch.bfloat16, device="cuda")
    wg = torch.zeros(4, 72, dtype=torch.bfloat16, device="cuda")
    q = torch.zeros(4, 128 * 72 // 2, dtype=torch.uint8, device="cuda")
    s = torch.full((4, 2048), 127, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.MoeError) as ei:
        m.moe_layer_forward_w4(x, wg, q, q, s, s)
    assert ei.value.code == binding.MOE_ERR_UNSUPPORTED
    ok = binding.MoeLayer(64, 64, 128, 4, 2, "bf16")
    with pytest.raises(binding.MoeError) as ei:        # rows not a multiple of 32
        ok.moe_quantize_mxfp4(torch.zeros(4, 48, 64, dtype=torch.bfloat16, device="cuda"))
    assert ei.value.code == binding.MOE_ERR_INVALID_ARG
    assert ok.lib.moe_mxfp4_scale_bytes(64, 640) == 2 * 2 * 512
    torch.cuda.synchronize()


@pytest.mark.parametrize("fmt", ["w8", "w4"])
def test_quantised_layer_T_zero_T_one_and_one_hot_routing(dev, fmt):
    """Degenerate batches through the quantised calls: no token, one token, and every token on the
    same two experts (all other experts idle, their weights poisoned)."""
    from oracle import quant_e4m3 as o8
    w = wl.CONFIGS["lm"].scaled(name="q_edge", T=300, D=128, F=256, E=8, k=2, gate_scale=1.0, zipf_s=0.0)
    inp = wl.make_inputs(w, with_ffn_bias=True)
    # a gate bias that decides the routing for every token: experts 5 and 2, in that order
    gb = torch.zeros(w.E, dtype=torch.float32)
    gb[5], gb[2] = 60.0, 40.0
    g = {k: (None if v is None else v.cuda()) for k, v in inp.items()}
    g["gate_bias"] = gb.cuda()
    m = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, "bf16")
    if fmt == "w8":
        q1, s1 = m.moe_quantize_e4m3(g["w1"])
        q2, s2 = m.moe_quantize_e4m3(g["w2"])
        fwd, oqm = m.moe_layer_forward_w8, o8
        deq = lambda t: torch.from_numpy(o8.dequantize(*o8.quantize(t.float().numpy().astype(np.float64))).astype(np.float32)).to(torch.bfloat16)
        poison = 0x7F
    else:
        q1, s1 = m.moe_quantize_mxfp4(g["w1"])
        q2, s2 = m.moe_quantize_mxfp4(g["w2"])
        fwd = m.moe_layer_forward_w4
        deq = lambda t: dequant_bf16(*oq.quantize(t.float().numpy().astype(np.float64)))
        poison = 0x77
    for e in range(w.E):
        if e not in (2, 5):
            q1[e] = poison
            q2[e] = poison
            if fmt == "w4":
                s1[e] = 254
                s2[e] = 254
    w1r, w2r = deq(inp["w1"]), deq(inp["w2"])
    for T in (0, 1, w.T):
        x = g["x"][:T].contiguous()
        r = m.empty_routing(T)
        y = fwd(x, g["wg"], q1, q2, s1, s2, g["gate_bias"], g["b1"], g["b2"], routing_out=r)
        torch.cuda.synchronize()
        assert y.shape == (T, w.D)
        if T == 0:
            assert int(r["counts"].sum()) == 0
            continue
        ridx = np.tile(np.array([[5, 2]], dtype=np.int32), (T, 1))
        np.testing.assert_array_equal(to_np(r["topk_idx"]), ridx)
        assert to_np(r["counts"]).tolist() == [0, 0, T, 0, 0, T, 0, 0]
        logits = orc.gate_logits(inp["x"][:T], inp["wg"], gb)
        _, rw = orc.topk(logits, w.k, True)
        ref = orc.layer_tokens(inp["x"][:T], w1r, w2r, ridx, rw, b1=inp["b1"], b2=inp["b2"])
        got = to_np(y)
        assert np.all(np.isfinite(got))
        err = norm_max_err(got, ref)
        say("  %s T=%d err=%.3e" % (fmt, T, err))
        assert err <= TOL["bf16"], err
