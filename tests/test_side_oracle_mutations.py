"""The pins of the Expert Buffering and placement oracles must be able to fail: each plausible
mistake is planted in a copy of the oracle's source, the copy is loaded as a module, and the
oracle's own pin tests are run against it -- at least one of them has to fail."""
import os
import types

import pytest

import test_expert_cache_oracle as pins_cache
import test_placement_oracle as pins_place
from test_quant_oracle_mutations import run_pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = {
    # name: (oracle file, pin module, attribute the pin module calls the oracle by, text to replace, replacement)
    "cache_first_in_first_out_inside_a_class": ("expert_cache.py", pins_cache, "ec",
                                                "return max(pool, key=lambda e: self.inserted[e])",
                                                "return min(pool, key=lambda e: self.inserted[e])"),
    "cache_active_residents_not_spared": ("expert_cache.py", pins_cache, "ec",
                                          "pool = idle if idle else residents", "pool = residents"),
    "cache_lru_by_insertion": ("expert_cache.py", pins_cache, "ec",
                               "return min(residents, key=lambda e: self.used.get(e, -1))",
                               "return min(residents, key=lambda e: self.inserted[e])"),
    "cache_belady_evicts_the_nearest": ("expert_cache.py", pins_cache, "ec",
                                        "return max(residents, key=next_use)", "return min(residents, key=next_use)"),
    "cache_stage_not_advanced": ("expert_cache.py", pins_cache, "ec",
                                 "stage = max(stage, stage_of[victim] + 1)", "stage = max(stage, stage_of[victim])"),
    "cache_hit_counted_as_miss": ("expert_cache.py", pins_cache, "ec", "self.hits += 1", "self.misses += 1"),
    "place_ascending_load_order": ("placement.py", pins_place, "pl",
                                   "order = sorted(range(E), key=lambda m: (-mu[m], m))",
                                   "order = sorted(range(E), key=lambda m: (mu[m], m))"),
    "place_correlation_sign": ("placement.py", pins_place, "pl",
                               "load += mu[m] + (corr_weight * S[a][m] if S is not None else 0.0)",
                               "load += mu[m] - (corr_weight * S[a][m] if S is not None else 0.0)"),
    "place_capacity_ignored": ("placement.py", pins_place, "pl", "if len(members[n]) >= cap:", "if False:"),
    "place_pearson_not_normalised": ("placement.py", pins_place, "pl",
                                     "S[a][m] = c / math.sqrt(ss[a] * ss[m])", "S[a][m] = c"),
    "place_max_load_is_the_mean": ("placement.py", pins_place, "pl", "worst = max(worst, mx)", "worst = mx"),
    "place_heaviest_device_first": ("placement.py", pins_place, "pl",
                                    "if best < 0 or load < best_load:", "if best < 0 or load > best_load:"),
}


def load_mutant(name):
    fname, pins, attr, old, new = MUTATIONS[name]
    text = open(os.path.join(ROOT, "oracle", fname)).read()
    assert text.count(old) >= 1, "mutation site for %s not found" % name
    mod = types.ModuleType("mutant_" + name)
    exec(compile(text.replace(old, new, 1), fname, "exec"), mod.__dict__)
    return mod, pins, attr


def run(pins, attr, oracle):
    # run_pins swaps the attribute `oq`; these pin modules use another name for the oracle
    saved = getattr(pins, attr)
    had = hasattr(pins, "oq")
    setattr(pins, "oq", oracle)
    setattr(pins, attr, oracle)
    try:
        return run_pins(pins, oracle)
    finally:
        setattr(pins, attr, saved)
        if not had:
            delattr(pins, "oq")


def test_pins_pass_on_the_unmodified_oracles():
    from oracle import expert_cache, placement
    assert run(pins_cache, "ec", expert_cache) == []
    assert run(pins_place, "pl", placement) == []


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name):
    mod, pins, attr = load_mutant(name)
    assert run(pins, attr, mod), "no pin noticed the planted mistake '%s'" % name
