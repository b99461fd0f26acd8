"""Pins for oracle.allocation (Sec. 3.2: per-layer densities by the Erdos-Renyi strategy)."""
import random

import pytest

from oracle import allocation as al

GPT2_SMALL_BLOCK = [(2304, 768), (768, 768), (3072, 768), (768, 3072)]   # (O, I)


def budget(shapes, dens):
    return sum(d * O * I for (O, I), d in zip(shapes, dens))


def solve_by_bisection(shapes, d):
    """Independent solve: the kept budget is monotone in eps, so bisect on eps."""
    target = d * sum(O * I for O, I in shapes)

    def kept(eps):
        return sum(min(1.0, eps * (O + I) / (O * I)) * O * I for O, I in shapes)

    lo, hi = 0.0, max(O * I / (O + I) for O, I in shapes)      # at hi every layer is dense
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if kept(mid) < target:
            lo = mid
        else:
            hi = mid
    return [min(1.0, hi * (O + I) / (O * I)) for O, I in shapes]


def test_hand_computed_block_at_ten_percent():
    # N = 1769472 + 589824 + 2 * 2359296 = 7077888, sum (I + O) = 12288,
    # eps = 0.1 * 7077888 / 12288 = 57.6
    d = al.erdos_renyi_density(GPT2_SMALL_BLOCK, 0.1)
    assert d[0] == pytest.approx(57.6 * 3072 / 1769472, rel=1e-14)      # 0.1
    assert d[1] == pytest.approx(0.15, rel=1e-14)
    assert d[2] == pytest.approx(0.09375, rel=1e-14)
    assert d[3] == pytest.approx(0.09375, rel=1e-14)


def test_hand_computed_saturating_pair():
    # 2 x 2 and 100 x 100 at d = 0.5: budget 5002; unsaturated eps = 5002 / 204 gives the
    # small layer 24.5 > 1, so it is dense and eps = (5002 - 4) / 200 = 24.99
    d = al.erdos_renyi_density([(2, 2), (100, 100)], 0.5)
    assert d[0] == 1.0
    assert d[1] == pytest.approx(24.99 * 200 / 10000, rel=1e-14)


def test_budget_is_conserved_and_matches_bisection():
    rng = random.Random(7)
    for case in range(200):
        shapes = [(rng.randint(1, 400), rng.randint(1, 400)) for _ in range(rng.randint(1, 9))]
        d = rng.choice([0.0, 0.02, 0.04, 0.1, 0.3, 0.5, 0.9, 0.99, 1.0, rng.random()])
        got = al.erdos_renyi_density(shapes, d)
        assert all(0.0 <= g <= 1.0 for g in got)
        total = sum(O * I for O, I in shapes)
        assert budget(shapes, got) == pytest.approx(d * total, rel=1e-12, abs=1e-9)
        want = solve_by_bisection(shapes, d)
        assert got == pytest.approx(want, rel=1e-9, abs=1e-12), (case, shapes, d)


def test_unsaturated_layers_share_one_eps():
    shapes = [(3, 5), (40, 60), (200, 100), (64, 64)]
    got = al.erdos_renyi_density(shapes, 0.3)
    eps = [g * O * I / (O + I) for (O, I), g in zip(shapes, got) if g < 1.0]
    assert len(eps) >= 2 and max(eps) - min(eps) < 1e-12 * max(eps)
    # a saturated layer would have asked for more than its size
    for (O, I), g in zip(shapes, got):
        if g == 1.0:
            assert eps[0] * (O + I) / (O * I) >= 1.0


def test_special_cases():
    assert al.erdos_renyi_density(GPT2_SMALL_BLOCK, 1.0) == [1.0] * 4
    assert al.erdos_renyi_density(GPT2_SMALL_BLOCK, 0.0) == [0.0] * 4
    same = al.erdos_renyi_density([(128, 64)] * 5, 0.37)
    assert same == pytest.approx([0.37] * 5, rel=1e-14)          # equal shapes: the network's density
    assert al.erdos_renyi_density([(10, 20)], 0.25) == pytest.approx([0.25], rel=1e-14)
    # smaller layers are kept denser
    d = al.erdos_renyi_density([(64, 64), (128, 128), (256, 256)], 0.1)
    assert d[0] > d[1] > d[2]
    # the order of the layers does not matter
    p = al.erdos_renyi_density([(256, 256), (64, 64), (128, 128)], 0.1)
    assert [p[1], p[2], p[0]] == pytest.approx(d, rel=1e-14)


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        al.erdos_renyi_density([], 0.5)
    with pytest.raises(ValueError):
        al.erdos_renyi_density([(0, 4)], 0.5)
    with pytest.raises(ValueError):
        al.erdos_renyi_density([(4, 4)], 1.5)
