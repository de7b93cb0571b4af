"""The library's cache management (moe_cache_policy_*, host logic, no GPU) against the oracle of
paper Sec. 6: every decision -- slot, victim, stage, hit / miss count -- must be identical."""
import json
import os
import random

import pytest

from oracle import expert_cache as ec
from paper_2303_06182_amd import binding

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "expert_cache_example.json")


def test_paper_example_through_the_c_abi():
    g = json.load(open(GOLD))
    pol = binding.CachePolicy(g["n_experts"], g["n_slots"])
    counts = [1 if e in g["active"] else 0 for e in range(g["n_experts"])]
    slot_of, stage_of, loads, n_stages = pol.step(counts)
    assert [l[0] for l in loads] == [1, 2, 3]
    assert loads[2][2] == g["victim_when_loading_3"]
    assert n_stages == 2 and stage_of == [-1, 0, 0, 1]
    hits, misses, held = pol.stats()
    assert (hits, misses) == (0, 3) and sorted(held) == g["residents_after_batch"]
    assert slot_of[0] == -1 and slot_of[3] == slot_of[2]     # expert 3 took expert 2's slot


@pytest.mark.parametrize("seed", range(12))
def test_policy_matches_oracle(seed):
    rng = random.Random(seed)
    E = rng.choice([3, 8, 16, 64, 128])
    slots = rng.randint(1, E)
    pol = binding.CachePolicy(E, slots)
    orc = ec.ExpertCache(slots, "paper")
    p_active = rng.choice([0.1, 0.3, 0.7])
    state = [rng.random() < p_active for _ in range(E)]
    for _ in range(40):
        state = [s if rng.random() < 0.7 else (rng.random() < p_active) for s in state]
        counts = [rng.randint(1, 9) if s else 0 for s in state]
        slot_of, stage_of, loads, n_stages = pol.step(counts)
        out = orc.step([e for e in range(E) if counts[e] > 0])
        assert n_stages == out["n_stages"]
        assert loads == [(l.expert, l.slot, l.victim, l.stage) for l in out["loads"]]
        assert slot_of == [out["slot_of"].get(e, -1) for e in range(E)]
        assert stage_of == [out["stage_of"].get(e, -1) for e in range(E)]
    hits, misses, held = pol.stats()
    assert (hits, misses) == (orc.hits, orc.misses)
    assert held == orc.slot_expert
    pol.reset()
    assert pol.stats() == (0, 0, [-1] * slots)


def test_bad_arguments():
    with pytest.raises(binding.MoeError):
        binding.CachePolicy(0, 1)
    with pytest.raises(binding.MoeError):
        binding.CachePolicy(4, 0)
    lib = binding.load_library()
    assert lib.moe_cache_policy_reset(None) == binding.MOE_ERR_INVALID_ARG
    assert lib.moe_layer_forward_buffered(None, None, None, None, None, None, None, 0, None, None, None, 0,
                                          None) == binding.MOE_ERR_INVALID_ARG
    assert lib.moe_expert_cache_bytes(None, 4) == binding.MOE_ERR_INVALID_ARG
