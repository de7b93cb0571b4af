"""GPU parity on seeded random shapes: T, D, F, E, k, bias, renormalisation and routing skew drawn
per case, through the fused layer call in every weight format (bf16, fp32, e4m3, mxfp4), routing
bit-exact and output within the format's bar against the fp64 oracle."""
import sys

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from oracle import quant_e4m3 as o8
from oracle import quant_mxfp4 as o4
from paper_2303_06182_amd import binding, workloads as wl
from helpers import RMS_TOL, TOL, guarded_inputs, norm_max_err, rms_rel_err, to_np

pytestmark = pytest.mark.gpu

FORMATS = ["bf16", "f32", "w8", "w4", "bf16"]


def draw_case(i):
    rng = np.random.default_rng(9000 + i)
    fmt = FORMATS[i % len(FORMATS)]
    E = int(rng.choice([1, 2, 3, 5, 8, 16, 37, 64, 130, 256]))
    k = int(rng.integers(1, min(E, 4) + 1))
    T = int(rng.choice([1, 2, 7, 33, 64, 100, 255, 256, 257, 700, 2049, 3000]))
    if fmt in ("w8", "w4"):
        D, F = 64 * int(rng.integers(1, 9)), 64 * int(rng.integers(1, 13))
    else:
        D, F = 8 * int(rng.integers(1, 50)), 8 * int(rng.integers(1, 80))
    return dict(i=i, fmt=fmt, T=T, D=D, F=F, E=E, k=k, zipf=float(rng.choice([0.0, 0.8, 1.5])),
                gs=float(rng.choice([1.0, 30.0, 100.0])), bias=bool(rng.integers(0, 2)), renorm=bool(rng.integers(0, 2)))


CASES = [draw_case(i) for i in range(30)]


def as_bf16(a64):
    return torch.from_numpy(a64.astype(np.float32)).to(torch.bfloat16)


@pytest.mark.parametrize("c", CASES, ids=["%d_%s" % (c["i"], c["fmt"]) for c in CASES])
def test_layer_forward_random_shape(c):
    print("random shape", c, flush=True)
    sys.stdout.flush()
    dtype = "f32" if c["fmt"] == "f32" else "bf16"
    w = wl.Workload("rnd%d" % c["i"], dtype, T=c["T"], D=c["D"], F=c["F"], E=c["E"], k=c["k"], zipf_s=c["zipf"],
                    zipf_c=0.5, gate_scale=c["gs"], seed=9000 + c["i"])
    inp, _ = guarded_inputs(w, with_ffn_bias=c["bias"])
    g = {a: (None if v is None else v.cuda()) for a, v in inp.items()}
    m = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, dtype, c["renorm"])
    r = m.empty_routing(w.T)
    w1r, w2r = inp["w1"], inp["w2"]
    if c["fmt"] == "w8":
        q1, s1 = m.moe_quantize_e4m3(g["w1"])
        q2, s2 = m.moe_quantize_e4m3(g["w2"])
        y = m.moe_layer_forward_w8(g["x"], g["wg"], q1, q2, s1, s2, g["gate_bias"], g["b1"], g["b2"], routing_out=r)
        w1r = as_bf16(o8.dequantize(*o8.quantize(inp["w1"].float().numpy().astype(np.float64))))
        w2r = as_bf16(o8.dequantize(*o8.quantize(inp["w2"].float().numpy().astype(np.float64))))
    elif c["fmt"] == "w4":
        q1, s1 = m.moe_quantize_mxfp4(g["w1"])
        q2, s2 = m.moe_quantize_mxfp4(g["w2"])
        y = m.moe_layer_forward_w4(g["x"], g["wg"], q1, q2, s1, s2, g["gate_bias"], g["b1"], g["b2"], routing_out=r)
        w1r = as_bf16(o4.dequantize(*o4.quantize(inp["w1"].float().numpy().astype(np.float64))))
        w2r = as_bf16(o4.dequantize(*o4.quantize(inp["w2"].float().numpy().astype(np.float64))))
    else:
        y = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"], g["b1"], g["b2"], routing_out=r)
    torch.cuda.synchronize()
    logits = orc.gate_logits(inp["x"], inp["wg"], inp["gate_bias"])
    ridx, rw = orc.topk(logits, w.k, c["renorm"])
    np.testing.assert_array_equal(to_np(r["topk_idx"]), ridx)
    rc, ro, rd, rs = orc.route(ridx, w.E)
    np.testing.assert_array_equal(to_np(r["counts"]), rc)
    np.testing.assert_array_equal(to_np(r["offsets"]), ro)
    np.testing.assert_array_equal(to_np(r["dst_row"]), rd)
    np.testing.assert_array_equal(to_np(r["src_tok"]), rs)
    ref = orc.layer_tokens(inp["x"], w1r, w2r, ridx, rw, b1=inp["b1"], b2=inp["b2"])
    got = to_np(y)
    assert np.all(np.isfinite(got))
    err, rms = norm_max_err(got, ref), rms_rel_err(got, ref)
    print("  err %.3e rms %.3e" % (err, rms), flush=True)
    assert err <= TOL[dtype], err
    assert rms <= RMS_TOL[dtype], rms
