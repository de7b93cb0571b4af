"""Pins of the Expert Buffering cache oracle (paper Sec. 6): the paper's worked example, textbook
special cases, invariants, and brute force on tiny traces."""
import itertools
import json
import os
import random

import pytest

from oracle import expert_cache as ec

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "expert_cache_example.json")


def random_trace(seed, n_experts, n_batches, p_active, sticky=0.7):
    """Temporally correlated activity: an expert keeps its state with probability `sticky`."""
    rng = random.Random(seed)
    state = [rng.random() < p_active for _ in range(n_experts)]
    trace = []
    for _ in range(n_batches):
        state = [s if rng.random() < sticky else (rng.random() < p_active) for s in state]
        trace.append([e for e in range(n_experts) if state[e]])
    return trace


def test_paper_worked_example():
    g = json.load(open(GOLD))
    c = ec.ExpertCache(g["n_slots"], "paper")
    out = c.step(g["active"])
    loads = [l.astuple() for l in out["loads"]]
    # experts 1 and 2 fill the two slots, then 3 replaces 2 (last in), not 1
    assert [l[1] for l in loads] == [1, 2, 3]
    assert [l[3] for l in loads] == [-1, -1, g["victim_when_loading_3"]]
    assert c.residents() == g["residents_after_batch"]
    assert g["kept"] in c.residents()
    # expert 2 ran before its slot was taken: expert 3 is one stage later
    assert out["stage_of"] == {1: 0, 2: 0, 3: 1}
    assert out["n_stages"] == 2
    # FIFO would have thrown out expert 1, the one needed first in the next batch
    f = ec.ExpertCache(g["n_slots"], "fifo")
    f.step(g["active"])
    assert f.residents() == [2, 3]


def test_inactive_residents_go_first_and_last_in_first():
    c = ec.ExpertCache(3, "paper")
    c.step([0, 1, 2])              # inserted in the order 0, 1, 2
    out = c.step([1, 5])           # 0 and 2 are idle; 2 entered last
    assert [(l.expert, l.victim) for l in out["loads"]] == [(5, 2)]
    assert out["stage_of"] == {1: 0, 5: 0}       # the victim did not run in this batch: no extra stage
    out = c.step([1, 5, 6])        # only 0 is idle
    assert [(l.expert, l.victim) for l in out["loads"]] == [(6, 0)]
    out = c.step([1, 5, 6, 7])     # nobody idle: last in among the active ones is 6
    assert [(l.expert, l.victim) for l in out["loads"]] == [(7, 6)]
    assert out["stage_of"][7] == out["stage_of"][6] + 1


def test_repeating_batch_lifo_beats_fifo():
    # the same three experts every batch, room for two: FIFO misses on every access,
    # the paper's policy keeps expert 0 for good (Sec. 6, "LIFO policy is better than FIFO")
    trace = [[0, 1, 2]] * 10
    fifo = ec.simulate(trace, 2, "fifo")
    paper = ec.simulate(trace, 2, "paper")
    assert fifo["misses"] == 30
    assert paper["per_batch_misses"][1:] == [2] * 9
    assert paper["misses"] < fifo["misses"]


@pytest.mark.parametrize("policy", ec.POLICIES)
def test_invariants(policy):
    for seed in range(6):
        trace = random_trace(seed, 12, 25, 0.35)
        for slots in (1, 2, 3, 5, 8, 12):
            r = ec.simulate(trace, slots, policy)
            assert r["hits"] + r["misses"] == sum(len(b) for b in trace)
            assert sum(r["per_batch_misses"]) == r["misses"] == len(r["loads"])
            assert len(r["residents"]) <= slots
            distinct = len(set(e for b in trace for e in b))
            assert r["misses"] >= distinct                     # every expert misses at least once
            if slots >= 12:
                assert r["misses"] == distinct                 # everything fits: cold misses only
            for l in r["loads"]:
                assert 0 <= l.slot < slots


def test_step_bookkeeping():
    for seed in range(4):
        trace = random_trace(100 + seed, 10, 20, 0.5)
        c = ec.ExpertCache(3, "paper")
        held = {}
        for b in trace:
            out = c.step(b)
            prev = -1
            for e in sorted(b):
                assert out["stage_of"][e] >= max(prev, 0)      # stages never decrease along the id order
                prev = out["stage_of"][e]
            for l in out["loads"]:
                if l.victim >= 0:
                    assert held.get(l.slot) == l.victim
                    if l.victim in out["stage_of"] and l.victim < l.expert:
                        assert l.stage > out["stage_of"][l.victim]
                held[l.slot] = l.expert
            # two experts that run in the same stage never share a slot
            seen = {}
            for e in sorted(b):
                key = (out["stage_of"][e], out["slot_of"][e])
                assert key not in seen, (key, e, seen[key])
                seen[key] = e


def test_belady_is_optimal_on_tiny_traces():
    for seed in range(12):
        trace = random_trace(200 + seed, 5, 5, 0.5, sticky=0.4)
        for slots in (1, 2, 3):
            b = ec.simulate(trace, slots, "belady")["misses"]
            assert b == ec.optimal_misses(trace, slots), (seed, slots)


def test_no_policy_beats_belady():
    for seed in range(8):
        trace = random_trace(300 + seed, 16, 40, 0.3)
        for slots in (2, 4, 8):
            best = ec.simulate(trace, slots, "belady")["misses"]
            for policy in ("paper", "fifo", "lru"):
                assert ec.simulate(trace, slots, policy)["misses"] >= best


def test_single_slot_and_empty_batches():
    r = ec.simulate([[3], [], [3], [4], [3, 4]], 1, "paper")
    assert r["per_batch_misses"] == [1, 0, 0, 1, 2]
    assert ec.simulate([[], []], 2, "paper")["miss_rate"] == 0.0
    with pytest.raises(ValueError):
        ec.ExpertCache(0)


def test_lru_and_fifo_by_hand():
    """Two slots, batches (1), (2), (1), (3), (1).  LRU: 3 replaces 2, because 1 was used in the third
    batch, and the last access of 1 hits.  FIFO: 3 replaces 1, the first to come in, and 1 then replaces 2."""
    trace = [[1], [2], [1], [3], [1]]
    lru = ec.simulate(trace, 2, "lru")
    assert [l.victim for l in lru["loads"]] == [-1, -1, 2]
    assert (lru["hits"], lru["misses"]) == (2, 3)
    fifo = ec.simulate(trace, 2, "fifo")
    assert [l.victim for l in fifo["loads"]] == [-1, -1, 1, 2]
    assert (fifo["hits"], fifo["misses"]) == (1, 4)
