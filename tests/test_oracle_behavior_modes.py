"""Pins for the Stage-1 variants (oracle.score_heads_modes) and the per-query-head budget mode
(CPU only): a hand-worked two-row head under every aggregation / ablation, reductions to the plain
functions, closed forms."""

from fractions import Fraction

import numpy as np
import pytest

import oracle
from conftest import read_golden
from paper_2508_15806_amd import workloads as wl

ROWS = np.array([[[[0.4, 0.3, 0.2, 0.1], [0.1, 0.5, 0.3, 0.1]]]], dtype=np.float32)   # [L=1, H=1, T=2, n=4]


def parse():
    out = []
    for line in read_golden("alg1_modes_worked.txt"):
        left, right = [p.strip() for p in line.split("|")]
        agg, a, b, c = left.split()
        out.append((agg, (a == "1", b == "1", c == "1"), [float(Fraction(t)) for t in right.split()]))
    return out


@pytest.mark.parametrize("ex", parse())
def test_worked_head(ex):
    agg, comps, want = ex
    acc, sc = oracle.score_heads_modes(ROWS, 1, 2, 2, aggregation=agg, components=comps)
    np.testing.assert_allclose(sc[0, 0], want, rtol=2e-7)      # the rows are fp32 values of the decimals
    np.testing.assert_allclose(acc[0, 0, :5], [1.1, 0.4, 0.2, 0.3, 2.0], rtol=2e-7)


def test_micro_with_all_components_is_score_heads():
    nr = wl.config4(L=2, H=3, T=5, n=512)
    acc5, sc5 = oracle.score_heads(nr.rows, nr.needle_start, nr.needle_len, nr.topk)
    acc8, sc8 = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk)
    assert np.array_equal(acc8[..., :5], acc5) and np.array_equal(sc8, sc5)
    assert (acc8[..., 7] == 0).all()


def test_macro_equals_micro_for_single_row_heads():
    nr = wl.config4(L=2, H=4, T=1, n=256)
    for comps in [(True, True, True), (True, True, False), (True, False, True)]:
        _, a = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk, "micro", comps)
        _, b = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk, "macro", comps)
        np.testing.assert_allclose(a, b, rtol=1e-15)


def test_macro_is_the_mean_of_row_scores_by_brute_force():
    nr = wl.config4(L=1, H=2, T=6, n=300)
    _, sc = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk, "macro")
    for h in range(2):
        sf = lg = 0.0
        for t in range(6):
            WO, WD, WS, _w = oracle.row_weights(nr.rows[0, h, t], nr.needle_start, nr.needle_len, nr.topk)
            sf += WO / (WO + WD) if WO + WD > 0 else 0.0
            lg += WO / (WO + WS) if WO + WS > 0 else 0.0
        sf /= 6
        lg /= 6
        inf = 2 * sf * lg / (sf + lg) if sf + lg > 0 else 0.0
        np.testing.assert_allclose(sc[0, h], [sf, lg, inf], rtol=1e-14)


def test_ablation_closed_forms():
    # without WS the logic score is 1 wherever the head hits the needle at all, and INF = 2 SF / (1 + SF)
    nr = wl.config4(L=1, H=6, T=4, n=400)
    _, full = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk)
    _, no_ws = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk, components=(True, True, False))
    _, no_wo = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk, components=(False, True, True))
    for h in range(6):
        sf = full[0, h, 0]
        assert no_ws[0, h, 0] == sf
        if sf > 0:
            assert no_ws[0, h, 1] == 1.0
            np.testing.assert_allclose(no_ws[0, h, 2], 2 * sf / (1 + sf), rtol=1e-15)
        assert (no_wo[0, h] == 0).all()
    # step 7 is the harmonic mean
    assert oracle.harmonic(0.5, 0.5) == 0.5 and oracle.harmonic(1.0, 0.0) == 0.0 and oracle.harmonic(0.0, 0.0) == 0.0
    np.testing.assert_allclose(oracle.harmonic(0.25, 0.75), 1 / (0.5 * (1 / 0.25 + 1 / 0.75)), rtol=1e-15)


def test_per_query_head_budgets():
    # hand-worked: L = 1, 4 query heads in 2 groups, avg 10, fixed 2: pool 32 over INF .5 .25 .25 0 -> 16 8 8 0
    got = oracle.allocate_budgets_per_query_head([[0.5, 0.25, 0.25, 0.0]], 4, 2, 10, 2)
    assert got == [[2 + 16 + 2 + 8, 2 + 8 + 2 + 0]]
    # G = 1: the plain rule
    inf = wl.inf_beta((9, 9), 3, 8).tolist()
    assert oracle.allocate_budgets_per_query_head(inf, 8, 8, 64, 16) == oracle.allocate_budgets(inf, 8, 8, 64, 16)
    # invariants: sums to avg * L * Hq, every KV head keeps at least G fixed parts
    inf = wl.inf_spiky((9, 10), 4, 16).tolist()
    got = oracle.allocate_budgets_per_query_head(inf, 16, 4, 100, 30)
    assert sum(map(sum, got)) == 100 * 4 * 16
    assert min(map(min, got)) >= 4 * 30
    # the group of the largest query-head scores gets the most within its layer
    for l in range(4):
        sums = [sum(inf[l][g * 4:(g + 1) * 4]) for g in range(4)]
        assert got[l].index(max(got[l])) == sums.index(max(sums))
