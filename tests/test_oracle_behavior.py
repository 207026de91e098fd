"""Pins for oracle/behavior.py (CPU only): hand-worked rows of Algorithm 1,
closed forms for uniform rows, the four-cell partition, brute force, and the
consistency of the harmonic-mean step with the values the paper prints."""

from fractions import Fraction

import numpy as np
import pytest

import oracle
from conftest import read_golden
from paper_2508_15806_amd import workloads as wl


def parse_rows():
    out = []
    for line in read_golden("alg1_worked_rows.txt"):
        wts, prm, cells, scores = [p.strip() for p in line.split("|")]
        wts = [float(v) for v in wts.split(",")]
        start, length, K = [int(t) for t in prm.split()]
        cells = [float(Fraction(t)) for t in cells.split()]
        scores = [float(Fraction(t)) for t in scores.split()]
        out.append((wts, start, length, K, cells, scores))
    return out


@pytest.mark.parametrize("ex", parse_rows())
def test_worked_rows(ex):
    wts, start, length, K, cells, scores = ex
    got = oracle.row_weights(np.array(wts, dtype=np.float64), start, length, K)
    np.testing.assert_allclose(got, cells, atol=1e-15)
    np.testing.assert_allclose(oracle.finalize_scores(*got[:3]), scores, atol=1e-15)


def brute_cells(row, start, length, K):
    order = sorted(range(len(row)), key=lambda j: (-float(row[j]), j))[:K]
    needle = set(range(start, start + length))
    WO = sum(float(row[j]) for j in order if j in needle)
    WD = sum(float(row[j]) for j in order if j not in needle)
    TNW = sum(float(row[j]) for j in needle)
    return WO, WD, max(0.0, TNW - WO)


def test_brute_force_random_rows():
    rng = np.random.default_rng(0)
    for trial in range(30):
        n = int(rng.integers(4, 64))
        row = rng.integers(0, 8, size=n).astype(np.float32)       # many ties
        row /= max(row.sum(), 1)
        length = int(rng.integers(1, n))
        start = int(rng.integers(0, n - length + 1))
        K = int(rng.integers(1, n + 1))
        WO, WD, WS, wide = oracle.row_weights(row, start, length, K)
        bWO, bWD, bWS = brute_cells(row, start, length, K)
        assert abs(WO - bWO) < 1e-12 and abs(WD - bWD) < 1e-12 and abs(WS - bWS) < 1e-12
        # the four cells partition the row's mass; WO + WD is the top-K mass
        assert abs(WO + WD + WS + wide - float(row.astype(np.float64).sum())) < 1e-12
        topk_mass = np.sort(row.astype(np.float64))[::-1][:K].sum()
        assert abs(WO + WD - topk_mass) < 1e-12


def test_uniform_row_closed_forms():
    n, K = 64, 8
    row = np.full(n, 1.0 / n, dtype=np.float32)
    for length in (4, 8, 16):
        WO, WD, WS, _ = oracle.row_weights(row, 0, length, K)     # top-K = [0, K) by the tie rule
        SF, LG, INF = oracle.finalize_scores(WO, WD, WS)
        assert abs(SF - min(length, K) / K) < 1e-12
        assert abs(LG - min(length, K) / length) < 1e-12
    WO, WD, WS, _ = oracle.row_weights(row, K, 8, K)              # needle after the top-K
    assert WO == 0.0 and oracle.finalize_scores(WO, WD, WS) == (0.0, 0.0, 0.0)


def test_needle_inside_topk_gives_lg_exactly_one():
    # Table 6 prints LG = 1.0 for head 0-31: this happens exactly when no needle mass is outside T_k
    rng = np.random.default_rng(1)
    row = rng.random(100).astype(np.float32) * 0.001
    row[40:44] = [0.2, 0.3, 0.1, 0.25]
    WO, WD, WS, _ = oracle.row_weights(row, 40, 4, 10)
    SF, LG, INF = oracle.finalize_scores(WO, WD, WS)
    assert WS == 0.0 and LG == 1.0 and 0 < SF < 1 and SF < INF < 1


def test_harmonic_mean_consistent_with_printed_tables():
    """Tables 7 and 8 list the same ten heads.  For each, some LG in (0, 1) must make the
    oracle's step 7 reproduce the printed INF from the printed SF, and that LG must lie below the
    smallest LG of Table 6 (none of the ten heads appears there)."""
    tabs = {"LG": {}, "SF": {}, "INF": {}}
    for line in read_golden("paper_tables_6_7_8.txt"):
        t, l, h, val = line.split()
        tabs[t][(int(l), int(h))] = float(val)
    assert set(tabs["SF"]) == set(tabs["INF"])
    lg_floor = min(tabs["LG"].values())
    for head, sf in tabs["SF"].items():
        target = tabs["INF"][head]
        lo, hi = 0.0, 1.0
        for _ in range(200):                                       # INF is increasing in LG
            mid = 0.5 * (lo + hi)
            inf = oracle.finalize_scores(1.0, 1.0 / sf - 1.0, 1.0 / mid - 1.0)[2] if mid > 0 else 0.0
            lo, hi = (mid, hi) if inf < target else (lo, mid)
        assert 0.0 < lo < lg_floor, (head, lo)
        assert sf < target < lo                                    # harmonic mean lies between its arguments
    # Table 8 is ranked by INF while Table 7 is ranked by SF: the two orders differ (14-31 vs 18-20),
    # which a score depending on SF alone could not produce
    by_sf = sorted(tabs["SF"], key=lambda k: -tabs["SF"][k])
    by_inf = sorted(tabs["INF"], key=lambda k: -tabs["INF"][k])
    assert by_sf != by_inf


def test_finalize_zero_over_zero():
    assert oracle.finalize_scores(0.0, 0.0, 0.0) == (0.0, 0.0, 0.0)
    assert oracle.finalize_scores(0.0, 1.0, 1.0) == (0.0, 0.0, 0.0)
    SF, LG, INF = oracle.finalize_scores(1.0, 1.0, 3.0)
    assert (SF, LG) == (0.5, 0.25) and abs(INF - 1.0 / 3.0) < 1e-15


def test_score_heads_micro_aggregation():
    nr = wl.config4(L=2, H=3, T=4, n=256, needle_len=8)
    acc, scores = oracle.score_heads(nr.rows, nr.needle_start, nr.needle_len, nr.topk)
    assert acc.shape == (2, 3, 5) and (acc[..., 4] == 4).all()
    for l in range(2):
        for h in range(3):
            cells = np.zeros(3)
            for t in range(4):
                cells += brute_cells(nr.rows[l, h, t], nr.needle_start, nr.needle_len, nr.topk)
            np.testing.assert_allclose(acc[l, h, :3], cells, rtol=1e-12, atol=1e-18)
            WO, WD, WS = cells
            sf = WO / (WO + WD) if WO + WD else 0.0
            assert abs(scores[l, h, 0] - sf) < 1e-12
    # rows sum to one, so the four cells sum to the row count
    np.testing.assert_allclose(acc[..., :4].sum(-1), acc[..., 4], rtol=1e-6)
    # accumulation across calls
    acc2, _ = oracle.score_heads(nr.rows, nr.needle_start, nr.needle_len, nr.topk, acc=acc.copy())
    np.testing.assert_allclose(acc2, 2 * acc, rtol=1e-15)
