"""Pins of the load-balancing oracle (paper Sec. 7): hand-worked cases, reductions, invariants and
exhaustive search on tiny inputs."""
import random

import pytest

from oracle import placement as pl


def activations(seed, E, B, skew=1.0, corr_pairs=()):
    """Random activation fractions: columns sum to 1; corr_pairs forces pairs of experts to move together."""
    rng = random.Random(seed)
    base = [(1.0 / (r + 1)) ** skew for r in range(E)]
    rng.shuffle(base)
    A = [[0.0] * B for _ in range(E)]
    for b in range(B):
        col = [base[m] * rng.lognormvariate(0.0, 0.6) for m in range(E)]
        for a, c in corr_pairs:
            col[c] = base[c] * col[a] / base[a]
        s = sum(col)
        for m in range(E):
            A[m][b] = col[m] / s
    return A


def test_greedy_by_hand():
    # average loads 0.4, 0.3, 0.2, 0.1 on two devices: 0.4 -> d0, 0.3 -> d1, 0.2 -> d1 (0.3 < 0.4),
    # 0.1 -> d0 (0.4 < 0.5): both devices end at 0.5
    A = [[0.4, 0.4], [0.3, 0.3], [0.2, 0.2], [0.1, 0.1]]
    assert pl.greedy(A, 2) == [0, 1, 1, 0]
    assert pl.loads(A, [0, 1, 1, 0], 2) == (0.5, 0.5)
    # a full device leaves the candidates: 6 experts, 3 devices of 2
    A = [[0.30], [0.25], [0.20], [0.15], [0.06], [0.04]]
    assert pl.greedy(A, 3) == [0, 1, 2, 2, 1, 0]
    # the original order (experts 0,1 | 2,3 | 4,5) is much worse
    assert pl.loads(A, [0, 0, 1, 1, 2, 2], 3)[0] == pytest.approx(0.55)
    assert pl.loads(A, pl.greedy(A, 3), 3)[0] == pytest.approx(0.35)


def test_ties_and_order():
    A = [[0.25, 0.25]] * 4
    assert pl.greedy(A, 2) == [0, 1, 0, 1]          # equal loads: lower expert first, lower device first
    with pytest.raises(ValueError):
        pl.greedy([[0.5], [0.3], [0.2]], 2)


def test_anticorrelation_separates_experts_that_fire_together():
    # experts 0 and 2 fire together, 1 and 3 fire together, the two groups alternate
    A = [[0.6, 0.0, 0.6, 0.0], [0.0, 0.6, 0.0, 0.6], [0.4, 0.0, 0.4, 0.0], [0.0, 0.4, 0.0, 0.4]]
    g = pl.greedy(A, 2)
    assert g == [0, 1, 0, 1]                         # by average load alone the pairs stay together
    assert pl.loads(A, g, 2) == (1.0, 1.0)           # one device takes the whole batch, every batch
    # expert 1 sees device 0 at 0.3 + 0.5 * (-1) = -0.2 < 0: experts that never fire together attract
    a = pl.anticorrelation(A, 2)
    assert a == [0, 0, 1, 1]
    assert pl.loads(A, a, 2) == (0.6, 0.6)


def test_anticorrelation_with_zero_weight_is_greedy():
    for seed in range(5):
        A = activations(seed, 16, 30)
        assert pl.anticorrelation(A, 4, 0.0) == pl.greedy(A, 4)


def test_pearson_basics():
    A = [[1.0, 2.0, 3.0], [2.0, 4.0, 6.0], [3.0, 2.0, 1.0], [5.0, 5.0, 5.0]]
    S = pl.pearson(A)
    assert S[0][1] == pytest.approx(1.0) and S[0][2] == pytest.approx(-1.0)
    assert S[3] == [0.0] * 4 and S[0][3] == 0.0      # a constant expert correlates with nobody
    for a in range(4):
        for m in range(4):
            assert S[a][m] == pytest.approx(S[m][a])


@pytest.mark.parametrize("seed", range(6))
def test_invariants_and_exhaustive_bound(seed):
    E, D, B = 8, 2, 12
    A = activations(seed, E, B, corr_pairs=((0, 1),))
    for place in (pl.greedy(A, D), pl.anticorrelation(A, D)):
        assert sorted(place.count(n) for n in range(D)) == [E // D] * D     # same number of experts everywhere
        mx, avg = pl.loads(A, place, D)
        assert 1.0 / D - 1e-12 <= avg <= mx <= 1.0 + 1e-12
        assert mx >= pl.best_max_load(A, D) - 1e-12                         # nobody beats the exhaustive optimum
    # on skewed loads the greedy placement beats the identity placement on the data it was built from
    ident = [m // (E // D) for m in range(E)]
    skewed = activations(seed, E, B, skew=2.0)
    assert pl.loads(skewed, pl.greedy(skewed, D), D)[1] <= pl.loads(skewed, ident, D)[1] + 1e-12
