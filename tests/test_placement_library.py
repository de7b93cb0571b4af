"""The library's placement functions (moe_placement_*, host logic, paper Sec. 7) against the oracle."""
import numpy as np
import pytest

from oracle import placement as pl
from paper_2303_06182_amd import binding
from test_placement_oracle import activations


def as_f32(A):
    """The library takes fp32 activations: give the oracle exactly those values."""
    return [[float(np.float32(v)) for v in row] for row in A]


@pytest.mark.parametrize("seed", range(8))
def test_placements_match_oracle(seed):
    E, D, B = [(8, 2, 10), (16, 4, 40), (64, 8, 60), (128, 8, 50)][seed % 4]
    A = as_f32(activations(seed, E, B, skew=1.0 + 0.3 * (seed % 3), corr_pairs=((0, 1), (2, 5))))
    g = binding.moe_placement_greedy(A, D)
    assert g == pl.greedy(A, D)
    a = binding.moe_placement_anticorrelation(A, D, 0.5)
    assert a == pl.anticorrelation(A, D, 0.5)
    for place in (g, a, [m % D for m in range(E)]):
        mx, av = binding.moe_placement_loads(A, place, D)
        omx, oav = pl.loads(A, place, D)
        assert mx == pytest.approx(omx, rel=1e-12) and av == pytest.approx(oav, rel=1e-12)


def test_train_on_one_half_evaluate_on_the_other():
    # the paper's protocol: placement from the first half of the data, loads on the second half
    E, D, B = 64, 8, 80
    A = as_f32(activations(7, E, B, skew=1.2))
    first = [row[:B // 2] for row in A]
    second = [row[B // 2:] for row in A]
    ident = [m // (E // D) for m in range(E)]
    g = binding.moe_placement_greedy(first, D)
    assert binding.moe_placement_loads(second, g, D)[1] < binding.moe_placement_loads(second, ident, D)[1]


def test_bad_arguments():
    with pytest.raises(binding.MoeError):
        binding.moe_placement_greedy([[0.5], [0.3], [0.2]], 2)          # 3 experts on 2 devices
    with pytest.raises(binding.MoeError):
        binding.moe_placement_loads([[0.5], [0.5]], [0, 2], 2)          # device id out of range
