"""GPU parity of the static-capacity baseline entry point against the static oracle
(same gate; first-empty-row slots in slot-major order; drops; zero padding)."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from paper_2303_06182_amd import binding, workloads as wl
from helpers import RMS_TOL, TOL, guarded_inputs, norm_max_err, rms_rel_err, to_np

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
MODES = [binding.MOE_STATIC_INDEXED, binding.MOE_STATIC_EINSUM]


def run_static(w, cap, mode, inp=None):
    if inp is None:
        inp, _ = guarded_inputs(w)
    g = {k: (None if v is None else v.cuda()) for k, v in inp.items()}
    m = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, w.dtype)
    r = m.empty_routing(w.T)
    y, dropped = m.moe_layer_forward_static(g["x"], g["wg"], g["w1"], g["w2"], cap, mode, g["gate_bias"], routing_out=r)
    torch.cuda.synchronize()
    ref = orc.static_layer(inp["x"], inp["wg"], inp["w1"], inp["w2"], w.k, cap, gate_bias=inp["gate_bias"])
    np.testing.assert_array_equal(to_np(r["topk_idx"]), ref["idx"])
    exp_rows = np.where(ref["keep"] == 1, ref["idx"] * cap + ref["slot"], -1)
    np.testing.assert_array_equal(to_np(r["dst_row"]), exp_rows)          # bit-exact slots and drops
    assert int(dropped[0]) == ref["dropped"]
    np.testing.assert_array_equal(to_np(r["counts"]), np.bincount(ref["idx"].ravel(), minlength=w.E))
    got = to_np(y)
    assert np.all(np.isfinite(got))
    # the einsum form rounds the gate weights to the storage type (one extra 2^-9 relative step in bf16)
    err = norm_max_err(got, ref["y"])
    assert err <= TOL[w.dtype], err
    return ref, got, m, g


CASES = [
    wl.CONFIGS["lm"].scaled(name="lm_s", T=600, D=128, F=256, E=8, gate_scale=100.0),
    wl.CONFIGS["skewed_large"].scaled(name="skew_s", T=1000, D=128, F=256, E=16),
    wl.CONFIGS["tiny_f32"].scaled(name="f32_s", T=200, D=64, F=128, gate_scale=100.0),
    wl.CONFIGS["lm"].scaled(name="odd_s", T=301, D=72, F=136, E=6, k=3, gate_scale=100.0, zipf_s=0.0),
]


@pytest.mark.parametrize("mode", MODES, ids=["indexed", "einsum"])
@pytest.mark.parametrize("w", CASES, ids=[c.name for c in CASES])
@pytest.mark.parametrize("cf", [0.5, 1.0, 2.0])
def test_static_layer_parity(w, mode, cf):
    print("static case", w.name, mode, cf, flush=True)
    cap = binding.moe_capacity(w.T, w.E, w.k, cf, binding.MOE_CAPACITY_SHARE)
    run_static(w, cap, mode)


@pytest.mark.parametrize("mode", MODES, ids=["indexed", "einsum"])
def test_static_equals_dynamic_when_nothing_is_dropped(mode):
    w = wl.CONFIGS["lm"].scaled(name="nodrop", T=500, D=128, F=256, E=8, gate_scale=100.0)
    inp, _ = guarded_inputs(w)
    dyn = orc.layer(inp["x"], inp["wg"], inp["w1"], inp["w2"], w.k, gate_bias=inp["gate_bias"])
    cap = int(dyn["counts"].max())
    ref, got, m, g = run_static(w, cap, mode, inp)
    assert ref["dropped"] == 0
    y_dyn = m.moe_layer_forward(g["x"], g["wg"], g["w1"], g["w2"], g["gate_bias"])
    torch.cuda.synchronize()
    assert norm_max_err(got, dyn["y"]) <= TOL[w.dtype]
    if mode == binding.MOE_STATIC_INDEXED:
        # same rows, same kernels, same order of the weighted sum: identical bits
        assert np.array_equal(to_np(y_dyn), got)


@pytest.mark.parametrize("mode", MODES, ids=["indexed", "einsum"])
def test_static_example_with_the_papers_dimensions(mode):
    """S = 6, E = 3, C = 0.5, top-1 (Sec. 5.1): capacity 3; the hand-worked assignment of
    tests/golden drops token 4, whose output row must be zero."""
    g = json.load(open(os.path.join(GOLDEN, "static_gating_example.json")))
    S, E, D, F = g["S"], g["E"], 8, 16
    cap = binding.moe_capacity(S, E, 1, g["C"], binding.MOE_CAPACITY_PAPER)
    assert cap == g["capacity"]
    x = np.zeros((S, D), dtype=np.float32)
    x[np.arange(S), g["assignment"]] = 1.0                   # logits = x . identity: the wanted expert wins
    x[:, E:] = np.random.default_rng(0).standard_normal((S, D - E)).astype(np.float32)
    wg = np.zeros((E, D), dtype=np.float32)
    wg[np.arange(E), np.arange(E)] = 1.0
    w1 = np.random.default_rng(1).standard_normal((E, F, D)).astype(np.float32)
    w2 = np.random.default_rng(2).standard_normal((E, D, F)).astype(np.float32)
    m = binding.MoeLayer(S, D, F, E, 1, "f32")
    r = m.empty_routing(S)
    y, dropped = m.moe_layer_forward_static(*[torch.from_numpy(a).cuda() for a in (x, wg, w1, w2)], cap, mode,
                                            routing_out=r)
    torch.cuda.synchronize()
    assert to_np(r["topk_idx"])[:, 0].tolist() == g["assignment"]
    slots = [(-1 if v < 0 else v % cap) for v in to_np(r["dst_row"])[:, 0].tolist()]
    assert slots == g["expected_slot"]
    assert int(dropped[0]) == len(g["expected_dropped_tokens"])
    got = to_np(y)
    for t in g["expected_dropped_tokens"]:
        assert np.all(got[t] == 0.0)
    ref = orc.static_layer(x, wg, w1, w2, 1, cap)
    assert norm_max_err(got, ref["y"]) <= 1e-5


def test_static_indexed_at_full_size_of_the_largest_workload():
    """skewed_large at its real size through the static baseline (index-moved rows, capacity factor 1.0 = 1024
    rows per expert: the configuration the benchmark times): slots and drops bit-exact for every assignment
    against the static oracle, the output on a token sample that holds fully dropped, half dropped and fully
    kept tokens."""
    w = wl.CONFIGS["skewed_large"]
    print("static full size", w, flush=True)
    inp, _ = guarded_inputs(w, device="cuda")
    m = binding.MoeLayer(w.T, w.D, w.F, w.E, w.k, w.dtype)
    cap = binding.moe_capacity(w.T, w.E, w.k, 1.0, binding.MOE_CAPACITY_SHARE)
    assert cap == 1024
    r = m.empty_routing(w.T)
    y, dropped = m.moe_layer_forward_static(inp["x"], inp["wg"], inp["w1"], inp["w2"], cap,
                                            binding.MOE_STATIC_INDEXED, inp["gate_bias"], routing_out=r)
    torch.cuda.synchronize()
    host = {k: (None if v is None else v.cpu()) for k, v in inp.items()}
    logits = orc.gate_logits(host["x"], host["wg"], host["gate_bias"])
    idx, gw = orc.topk(logits, w.k)
    slot, keep, n_dropped = orc.static_slots(idx, w.E, cap)
    np.testing.assert_array_equal(to_np(r["topk_idx"]), idx)
    np.testing.assert_array_equal(to_np(r["dst_row"]), np.where(keep == 1, idx * cap + slot, -1))
    assert int(dropped[0]) == n_dropped and n_dropped > w.T // 2      # the skewed gate overflows the hot experts
    kept = keep.sum(axis=1)
    rng = np.random.default_rng(7)
    tokens = np.concatenate([rng.choice(np.nonzero(kept == c)[0], size=min(700, int((kept == c).sum())), replace=False)
                             for c in (0, 1, 2)])
    # every expert's last kept row (slot cap - 1, or its last row when it is not full)
    last = {}
    for t, j in zip(*np.nonzero(keep == 1)):
        last[int(idx[t, j])] = int(t)
    tokens = np.union1d(tokens, np.array(sorted(last.values()))).astype(np.int32)
    ref = orc.layer_tokens(host["x"], host["w1"], host["w2"], idx, gw, tokens=tokens, keep=keep)
    got = to_np(y)[tokens]
    assert np.all(np.isfinite(to_np(y)))
    assert np.all(got[kept[tokens] == 0] == 0.0)                      # a fully dropped token leaves the layer as zero
    err, rms = norm_max_err(got, ref), rms_rel_err(got, ref)
    print("  static full size: dropped %d of %d, compared %d tokens, err %.3e rms %.3e" %
          (n_dropped, w.k * w.T, tokens.size, err, rms), flush=True)
    assert err <= TOL[w.dtype] and rms <= RMS_TOL[w.dtype]
    del m, inp, y
    torch.cuda.empty_cache()


def test_static_workspace_and_argument_errors():
    m = binding.MoeLayer(64, 64, 128, 8, 2, "bf16")
    n_idx = m.moe_static_workspace_bytes(64, 16, binding.MOE_STATIC_INDEXED)
    n_ein = m.moe_static_workspace_bytes(64, 16, binding.MOE_STATIC_EINSUM)
    assert 0 < n_idx < n_ein
    with pytest.raises(binding.MoeError):
        m.moe_static_workspace_bytes(64, 0, binding.MOE_STATIC_INDEXED)
    with pytest.raises(binding.MoeError):
        m.moe_static_workspace_bytes(64, 16, 9)
    w = wl.CONFIGS["lm"].scaled(T=64, D=64, F=128, E=8, zipf_s=0.0)
    g = {k: (None if v is None else v.cuda()) for k, v in wl.make_inputs(w).items()}
    with pytest.raises(binding.MoeError) as e:
        m.moe_layer_forward_static(g["x"], g["wg"], g["w1"], g["w2"], 16, binding.MOE_STATIC_EINSUM,
                                   workspace=torch.empty(n_idx // 2, dtype=torch.uint8, device="cuda"))
    assert e.value.code == binding.MOE_ERR_WORKSPACE
    torch.cuda.synchronize()
