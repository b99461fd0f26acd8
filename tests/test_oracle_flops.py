"""Pins for oracle.flops and oracle.attention_mask (App. "FLOP Calculation", Sec. 3.3)."""
import numpy as np
import pytest

from oracle import attention_mask as am
from oracle import flops as fl
from oracle import schedule as sc

VOCAB = 50304       # the public hyper-parameters' code base pads GPT-2's 50257 to a multiple of 64


def test_main_results_table_flops_column(golden):
    for row, n_layers, n_embd, S, q, printed in golden("table3_flops.txt"):
        n_embd = int(n_embd)
        got = fl.transformer(1024, n_embd, 4 * n_embd, VOCAB, int(n_layers), float(S), float(q))
        assert round(got["total"] / 1e9, 1) == float(printed), row


def test_fully_connected_terms_are_eq1_times_tokens():
    L, E, F, V, n = 1024, 768, 3072, VOCAB, 12
    S = 0.8
    t = fl.transformer(L, E, F, V, n, S, 1.0)
    block = [(3 * E, E), (E, E), (F, E), (E, F)]
    per_token = fl.fc_forward(block * n + [(V, E)], [S] * (4 * n + 1))
    fc = n * (t["kqv"] + t["proj"] + t["ffw1"] + t["ffw2"]) + t["lm"]
    assert fc == pytest.approx(L * per_token, rel=1e-14)
    assert t["forward"] == pytest.approx(fc + n * (t["scores"] + t["reduce"]), rel=1e-14)
    assert t["backward"] == 2 * t["forward"] and t["total"] == 3 * t["forward"]


def test_eq1_small_brute_force():
    # a dense O x I layer: every output is a dot product of I terms, I multiplies and
    # I - 1 adds
    for O, I in [(1, 1), (3, 5), (7, 2)]:
        assert fl.fc_forward([(O, I)], [0.0]) == O * (I + I - 1)
    assert fl.fc_forward([(4, 8), (2, 4)], [0.5, 0.25]) == 0.5 * 15 * 4 + 0.75 * 7 * 2


def test_attention_terms_count_multiply_adds_of_both_products():
    # scores: L x L dot products of length N_embd over all heads together (2 flops per
    # term); the second product has the same size
    t = fl.transformer(16, 8, 32, 100, 1, 0.0, 1.0)
    assert t["scores"] == 2 * 16 * 16 * 8 and t["reduce"] == t["scores"]
    half = fl.transformer(16, 8, 32, 100, 1, 0.0, 0.5)
    assert half["scores"] == t["scores"] / 2 and half["kqv"] == t["kqv"]


def test_mst_average_over_the_schedule_lies_near_a_quarter_of_dense():
    # Sec. 4 speaks of a FLOP reduction of about four times (219.4 G printed); with the
    # attention dense once the weights are, this reading of the schedule gives 226 G.
    cfg = sc.ScheduleCfg()
    dense = fl.transformer(1024, 768, 3072, VOCAB, 12, 0.0, 1.0)["total"]
    steps = 140000
    edges = sorted({0, steps} | {k * 2000 for k in range(0, 6)} | {110000 + k * 2000 for k in range(0, 6)})
    acc = 0.0
    for a, b in zip(edges, edges[1:]):
        d = sc.density(cfg, a)
        q = 1.0 if d >= 1.0 else 0.2203
        acc += (b - a) * fl.transformer(1024, 768, 3072, VOCAB, 12, 1.0 - d, q)["total"]
    avg = acc / steps
    assert 3.7 < dense / avg < 4.1
    assert avg / 1e9 == pytest.approx(226.2, abs=0.1)


def test_q_atten_table(golden):
    for stride, percent in golden("q_atten.txt"):
        assert round(100.0 * am.q_atten(1024, int(stride)), 2) == float(percent)


@pytest.mark.parametrize("L,l", [(1, 1), (7, 1), (9, 3), (16, 4), (33, 8), (20, 50)])
def test_mask_against_the_set_definition(L, l):
    m = am.strided_mask(L, l)
    for i in range(L):
        want = set(range(max(i - l + 1, 0), i + 1)) | {j for j in range(i + 1) if (i - j) % l == 0}
        assert set(np.nonzero(m[i])[0].tolist()) == want
    assert not np.triu(m, 1).any()                  # causal
    assert m.diagonal().all()                       # every position sees itself


def test_mask_row_at_the_figure_stride_three():
    # stride 3 as in the figure: row 7 sees the window 5, 6, 7 and the strided 1, 4
    m = am.strided_mask(10, 3)
    assert np.nonzero(m[7])[0].tolist() == [1, 4, 5, 6, 7]


def test_mask_count_closed_form():
    # row i keeps min(i + 1, l) window positions and floor(i / l) strided ones beyond the
    # window's own multiple (j = i)
    for L, l in [(1024, 128), (1024, 256), (100, 7), (64, 64), (64, 100)]:
        want = sum(min(i + 1, l) + i // l for i in range(L))
        assert int(am.strided_mask(L, l).sum(dtype=np.int64)) == want


def test_window_covering_the_sequence_is_the_causal_triangle():
    assert int(am.strided_mask(32, 32).sum()) == 32 * 33 // 2
    assert int(am.strided_mask(32, 1000).sum()) == 32 * 33 // 2
