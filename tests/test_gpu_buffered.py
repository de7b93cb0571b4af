"""Expert Buffering on the GPU (paper Sec. 6): moe_layer_forward_buffered must give the plain
call's result bit for bit while its cache behaves exactly like the oracle's."""
import sys

import numpy as np
import pytest
import torch

from oracle import expert_cache as ec
from oracle import moe_oracle as orc
from paper_2303_06182_amd import binding, workloads as wl
from helpers import TOL, norm_max_err, to_np

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load_library()
    return torch.device("cuda:0")


def run_trace(w, slots_list, n_steps=8, rho=0.8, with_bias=False):
    inp = wl.make_inputs(w, with_ffn_bias=with_bias)
    g = {k: (None if v is None else v.cuda()) for k, v in inp.items()}
    hw1, hw2 = inp["w1"].pin_memory(), inp["w2"].pin_memory()
    xs = [x.cuda() for x in wl.decode_steps(w, n_steps, rho)]
    layer = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, w.dtype)
    expert_bytes = 2 * w.F * w.D * (2 if w.dtype == "bf16" else 4)
    ref, trace = [], []
    for x in xs:
        r = layer.empty_routing(w.T)
        y = layer.moe_layer_forward(x, g["wg"], g["w1"], g["w2"], g["gate_bias"], g["b1"], g["b2"], routing_out=r)
        torch.cuda.synchronize()
        ref.append((y.clone(), r["dst_row"].clone(), r["topk_w"].clone()))
        trace.append(np.nonzero(to_np(r["counts"]))[0].tolist())
    for slots in slots_list:
        say("buffered", w.name, "slots", slots, "active per step", [len(t) for t in trace])
        cache = binding.ExpertCache(layer, slots, hw1, hw2)
        for rep in range(2):               # second pass: after reset the cache must behave the same
            for i, x in enumerate(xs):
                r = layer.empty_routing(w.T)
                y = cache.moe_layer_forward_buffered(x, g["wg"], g["gate_bias"], g["b1"], g["b2"], routing_out=r)
                torch.cuda.synchronize()
                assert torch.equal(y, ref[i][0]), "step %d, %d slots" % (i, slots)
                assert torch.equal(r["dst_row"], ref[i][1]) and torch.equal(r["topk_w"], ref[i][2])
            sim = ec.simulate(trace, slots, "paper")
            st = cache.stats()
            assert (st["hits"], st["misses"]) == (sim["hits"], sim["misses"])
            assert st["bytes_copied"] == sim["misses"] * expert_bytes
            assert st["stages"] >= len([t for t in trace if t])
            cache.reset()
        del cache
    return inp, xs, ref, trace


def test_buffered_equals_plain_bf16(dev):
    w = wl.CONFIGS["mt_decoder"].scaled(name="dec_small", T=24, D=128, F=256, E=16)
    inp, xs, ref, trace = run_trace(w, [1, 2, 5, 16])
    # and the plain call itself against the oracle on the last step
    x = xs[-1].cpu()
    logits = orc.gate_logits(x, inp["wg"], inp["gate_bias"])
    idx, gw = orc.topk(logits, w.k)
    y_ref = orc.layer_tokens(x, inp["w1"], inp["w2"], idx, gw)
    assert norm_max_err(to_np(ref[-1][0]), y_ref) <= TOL["bf16"]


def test_buffered_equals_plain_f32_with_biases(dev):
    w = wl.CONFIGS["tiny_f32"].scaled(name="f32_small", T=20, D=64, F=128, E=12)
    run_trace(w, [1, 3, 12], n_steps=5, with_bias=True)


def test_buffered_many_tokens_and_skew(dev):
    # every expert active, more experts than slots: the batch runs in several stages
    w = wl.CONFIGS["lm"].scaled(name="lm_small", T=2000, D=256, F=512, E=16)
    run_trace(w, [3, 16], n_steps=3)


def test_buffered_large_tiles(dev):
    # stages of three experts with 3000 rows each: 36 row tiles x 13 column tiles per stage, i.e. the 256-row
    # tiles' main launch reads its weights through the slot table; bit-identical to the resident call
    w = wl.CONFIGS["mt_encoder"].scaled(name="enc_mid", T=12000, D=256, F=3328, E=8)
    run_trace(w, [3, 8], n_steps=2)


def test_buffered_empty_batch_and_errors(dev):
    w = wl.CONFIGS["mt_decoder"].scaled(name="dec_small", T=8, D=64, F=128, E=8)
    inp = wl.make_inputs(w)
    layer = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, w.dtype)
    cache = binding.ExpertCache(layer, 2, inp["w1"].pin_memory(), inp["w2"].pin_memory())
    y = cache.moe_layer_forward_buffered(inp["x"].cuda()[:0], inp["wg"].cuda())
    assert y.shape[0] == 0 and cache.stats()["misses"] == 0
    other = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, w.dtype)
    with pytest.raises(binding.MoeError):
        # the cache was created for another handle
        binding._check(other.lib.moe_layer_forward_buffered(
            other.h, cache.c, binding._ptr(inp["x"].cuda()), binding._ptr(inp["wg"].cuda()), None, None, None, w.T,
            binding._ptr(torch.empty((w.T, w.D), dtype=torch.bfloat16, device="cuda")), None, *other._ws(),
            binding._stream()))
    with pytest.raises(binding.MoeError):
        binding.ExpertCache(layer, 0, inp["w1"].pin_memory(), inp["w2"].pin_memory())


@pytest.mark.parametrize("wbits", [8, 4])
def test_buffered_quantised_weights_equal_the_resident_call(dev, wbits):
    """The cache over e4m3 / e2m1 expert weights: bit for bit the result of moe_layer_forward_w8 / _w4
    with all experts resident (itself checked against the oracle elsewhere), the oracle's hit / miss
    counts, and half / a quarter of the bytes over the host link."""
    w = wl.CONFIGS["mt_decoder"].scaled(name="buf_q%d" % wbits, T=48, D=256, F=512, E=32)
    inp = wl.make_inputs(w, with_ffn_bias=True)
    g = {k: (None if v is None else v.cuda()) for k, v in inp.items()}
    xs = [x.cuda() for x in wl.decode_steps(w, 6, 0.8)]
    layer = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, w.dtype)
    if wbits == 8:
        q1, s1 = layer.moe_quantize_e4m3(g["w1"])
        q2, s2 = layer.moe_quantize_e4m3(g["w2"])
        fwd = layer.moe_layer_forward_w8
    else:
        q1, s1 = layer.moe_quantize_mxfp4(g["w1"])
        q2, s2 = layer.moe_quantize_mxfp4(g["w2"])
        fwd = layer.moe_layer_forward_w4
    torch.cuda.synchronize()
    hq1, hq2 = q1.cpu().pin_memory(), q2.cpu().pin_memory()
    expert_bytes = 2 * w.F * w.D * wbits // 8
    ref, trace = [], []
    for x in xs:
        r = layer.empty_routing(w.T)
        y = fwd(x, g["wg"], q1, q2, s1, s2, g["gate_bias"], g["b1"], g["b2"], routing_out=r)
        torch.cuda.synchronize()
        ref.append(y.clone())
        trace.append(np.nonzero(to_np(r["counts"]))[0].tolist())
    # the device copies of the quantised weights are not needed any more: the cache must not depend on them
    q1.fill_(0x7F)
    q2.fill_(0x7F)
    for slots in (4, 12, 32):
        say("buffered q%d" % wbits, "slots", slots, "active per step", [len(t) for t in trace])
        cache = binding.ExpertCache(layer, slots, hq1, hq2, wbits, s1, s2)
        for i, x in enumerate(xs):
            y = cache.moe_layer_forward_buffered(x, g["wg"], g["gate_bias"], g["b1"], g["b2"])
            torch.cuda.synchronize()
            assert torch.equal(y, ref[i]), "step %d, %d slots" % (i, slots)
        sim = ec.simulate(trace, slots, "paper")
        st = cache.stats()
        assert (st["hits"], st["misses"]) == (sim["hits"], sim["misses"])
        assert st["bytes_copied"] == sim["misses"] * expert_bytes
        del cache
