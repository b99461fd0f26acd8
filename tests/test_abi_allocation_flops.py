"""Host arithmetic of the library against the oracle: per-layer densities (Sec. 3.2),
FLOP counts (App. "FLOP Calculation") and the size of the strided pattern (Sec. 3.3)."""
import random

import numpy as np
import pytest

import paper_2408_11746_amd as mst
from oracle import allocation as oal
from oracle import attention_mask as oam
from oracle import flops as ofl

GPT2 = {"small": (768, 12), "medium": (1024, 24), "large": (1280, 36)}


def block(E):
    return [(3 * E, E), (E, E), (4 * E, E), (E, 4 * E)]


def test_erdos_renyi_matches_oracle():
    rng = random.Random(11)
    cases = [(block(768), d) for d in (0.04, 0.1, 0.24736, 0.53152, 0.9, 1.0, 0.0)]
    cases += [(block(E) * n + [(50304, E)], d) for E, n in GPT2.values() for d in (0.04, 0.2, 0.7)]
    for _ in range(300):
        shapes = [(rng.randint(1, 500), rng.randint(1, 500)) for _ in range(rng.randint(1, 12))]
        cases.append((shapes, rng.choice([rng.random(), 0.02, 0.5, 0.97, 0.999])))
    for shapes, d in cases:
        got = mst.mst_erdos_renyi_density(shapes, d)
        want = oal.erdos_renyi_density(shapes, d)
        assert got == pytest.approx(want, rel=1e-12, abs=1e-15), (shapes, d)
        assert [g == 1.0 for g in got] == [w == 1.0 for w in want] or max(
            abs(g - w) for g, w in zip(got, want)) < 1e-12


def test_erdos_renyi_rejects_bad_arguments():
    with pytest.raises(mst.MstError):
        mst.mst_erdos_renyi_density([], 0.5)
    with pytest.raises(mst.MstError):
        mst.mst_erdos_renyi_density([(4, 0)], 0.5)
    with pytest.raises(mst.MstError):
        mst.mst_erdos_renyi_density([(4, 4)], -0.1)
    with pytest.raises(mst.MstError):
        mst.mst_erdos_renyi_density([(4, 4)], float("nan"))


def test_densities_feed_the_count_rule_and_keep_the_budget():
    # the integer targets of the layers add up to the network's budget within one per layer
    shapes = block(768) * 12
    for d in (0.04, 0.10144, 0.53152):
        dens = mst.mst_erdos_renyi_density(shapes, d)
        targets = [mst.mst_update_counts(O * I, O * I, dl, 0.3, 0.25)["nnz_after"] for (O, I), dl in zip(shapes, dens)]
        total = sum(O * I for O, I in shapes)
        assert abs(sum(targets) - d * total) <= 0.5 * len(shapes) + 1e-6


def test_flops_match_oracle():
    rng = random.Random(5)
    for _ in range(200):
        shapes = [(rng.randint(1, 4000), rng.randint(1, 4000)) for _ in range(rng.randint(1, 10))]
        dens = [rng.random() for _ in shapes]
        got = mst.mst_flops_fc_forward(shapes, dens)
        assert got == pytest.approx(ofl.fc_forward(shapes, [1.0 - d for d in dens]), rel=1e-13)
    for E, n in GPT2.values():
        for d, q in [(1.0, 1.0), (0.2, 1.0), (0.04, 0.2203), (0.5, 0.1207)]:
            got = mst.mst_flops_transformer(1024, E, 4 * E, 50304, n, d, q)
            want = ofl.transformer(1024, E, 4 * E, 50304, n, 1.0 - d, q)
            for k, v in want.items():
                assert got[k] == pytest.approx(v, rel=1e-13), (E, d, q, k)
    with pytest.raises(mst.MstError):
        mst.mst_flops_transformer(0, 768, 3072, 50304, 12, 1.0, 1.0)
    with pytest.raises(mst.MstError):
        mst.mst_flops_transformer(1024, 768, 3072, 50304, 12, 1.5, 1.0)
    with pytest.raises(mst.MstError):
        mst.mst_flops_fc_forward([(4, 4)], [2.0])


def test_flops_reproduce_the_results_table(golden):
    for row, n_layers, n_embd, S, q, printed in golden("table3_flops.txt"):
        E = int(n_embd)
        got = mst.mst_flops_transformer(1024, E, 4 * E, 50304, int(n_layers), 1.0 - float(S), float(q))
        assert round(got["total"] / 1e9, 1) == float(printed), row


def test_strided_count_matches_oracle_and_table(golden):
    for L in list(range(1, 40)) + [64, 100, 257]:
        for l in [1, 2, 3, 5, 8, 16, 31, 64, 300]:
            want = int(oam.strided_mask(L, l).sum(dtype=np.int64))
            assert mst.mst_strided_attention_count(L, l) == want, (L, l)
    for stride, percent in golden("q_atten.txt"):
        c = mst.mst_strided_attention_count(1024, int(stride))
        assert round(100.0 * c / 1024 ** 2, 2) == float(percent)
    assert mst.mst_strided_attention_count(32768, 256) == sum(min(i + 1, 256) + i // 256 for i in range(32768))
    with pytest.raises(mst.MstError):
        mst.mst_strided_attention_count(0, 4)
    with pytest.raises(mst.MstError):
        mst.mst_strided_attention_count(4, 0)
