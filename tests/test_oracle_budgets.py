"""Pins for oracle/budgets.py (CPU only): hand-worked capacity maps stored under
tests/golden, the closed forms of Algorithm 2, and the invariants the
compression pass relies on."""

from fractions import Fraction

import numpy as np
import pytest

import oracle
from conftest import read_golden
from paper_2508_15806_amd import workloads as wl


def parse_examples():
    out = []
    for line in read_golden("budget_worked_examples.txt"):
        mode, dims, inf, caps = [p.strip() for p in line.split("|")]
        L, Hq, Hkv, avg, fixed = [int(t) for t in dims.split()]
        inf = [[float(v) for v in row.split(",")] for row in inf.split(";")]
        caps = [[int(v) for v in row.split(",")] for row in caps.split(";")]
        out.append((mode, L, Hq, Hkv, avg, fixed, inf, caps))
    return out


@pytest.mark.parametrize("ex", parse_examples())
def test_worked_examples(ex):
    mode, L, Hq, Hkv, avg, fixed, inf, caps = ex
    fn = oracle.allocate_budgets if mode == "exact" else oracle.allocate_budgets_literal
    assert fn(inf, Hq, Hkv, avg, fixed) == caps


def test_fixed_from_beta():
    # b_c (1 - 1/beta) with the paper's beta = 1.351 (Table 1)
    assert oracle.fixed_from_beta(64, 1.351) == 17      # 16.63
    assert oracle.fixed_from_beta(128, 1.351) == 33     # 33.26
    assert oracle.fixed_from_beta(128, 4.0 / 3.0) == 32
    assert oracle.fixed_from_beta(512, 8.0 / 7.0) == 64


def test_literal_closed_forms():
    # uniform INF: every head gets b_fixed + (b_c/beta) (0.01 + 1/L)  (Algorithm 2, steps 1-7)
    L, H, avg, fixed = 4, 8, 100, 20
    caps = oracle.allocate_budgets_literal([[0.3] * H] * L, H, H, avg, fixed)
    expect = int(np.floor(20 + 80 * (0.01 + 1.0 / L) + 0.5))
    assert caps == [[expect] * H] * L
    # sum of the un-rounded dynamic parts = B_total (0.01 + sum_i L_i^2)
    rng = np.random.default_rng(0)
    inf = rng.random((6, 4))
    tot = inf.sum()
    Li = inf.sum(axis=1) / tot
    B_total = 80 * 6 * 4
    dyn = B_total * (0.01 + Li)[:, None] * inf / tot
    assert abs(dyn.sum() - B_total * (0.01 + (Li ** 2).sum())) < 1e-9
    lit = np.array(oracle.allocate_budgets_literal(inf.tolist(), 4, 4, 100, 20))
    assert np.abs(lit - (20 + dyn)).max() <= 0.5 + 1e-9


def exact_reference(inf, avg, fixed):
    """Independent statement of the EXACT rule for G = 1 using Fractions: quotas
    from exact rationals of the 2^-30-quantised INF, Hamilton apportionment."""
    L, H = len(inf), len(inf[0])
    x = [[int(np.floor(v * 2 ** 30 + 0.5)) for v in row] for row in inf]
    A = [sum(r) for r in x]
    T = sum(A)
    pool = (avg - fixed) * L * H

    def hamilton(total, w):
        if sum(w) == 0:
            w = [1] * len(w)
        q = [Fraction(total) * Fraction(wi, sum(w)) for wi in w]
        fl = [int(qi) for qi in q]
        spare = total - sum(fl)
        while spare:
            best = max(range(len(w)), key=lambda i: (q[i] - fl[i], -i))
            fl[best] += 1
            q[best] = Fraction(fl[best])       # its remainder is used up
            spare -= 1
        return fl

    lw = [Fraction(1, 100) + Fraction(a, T) for a in A] if T else [Fraction(1)] * L
    den = 1
    for f in lw:
        den *= f.denominator
    lw_int = [int(f * den) for f in lw]
    lp = hamilton(pool, lw_int)
    return [[fixed + dyn for dyn in hamilton(lp[l], x[l])] for l in range(L)]


def test_exact_matches_independent_fraction_reference():
    rng = np.random.default_rng(1)
    for trial in range(10):
        L, H = int(rng.integers(1, 5)), int(rng.integers(1, 6))
        inf = rng.random((L, H)).round(3).tolist()
        avg = int(rng.integers(1, 300))
        fixed = int(rng.integers(0, avg + 1))
        assert oracle.allocate_budgets(inf, H, H, avg, fixed) == exact_reference(inf, avg, fixed)


@pytest.mark.parametrize("seed", range(6))
def test_exact_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    L, Hkv, G = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.choice([1, 2, 4]))
    Hq = Hkv * G
    inf = wl.inf_spiky((seed, 5), L, Hq) if seed % 2 else rng.random((L, Hq))
    avg = int(rng.integers(8, 1025))
    fixed = int(rng.integers(0, avg + 1))
    caps = np.array(oracle.allocate_budgets(inf.tolist(), Hq, Hkv, avg, fixed))
    assert caps.shape == (L, Hkv)
    assert caps.sum() == avg * L * Hkv                       # integers summing exactly to the total
    assert (caps >= fixed).all()                             # every head keeps its fixed part
    means = inf.reshape(L, Hkv, G).mean(axis=2)
    for l in range(L):                                       # dynamic share monotone in INF within a layer
        for a in range(Hkv):
            for b in range(Hkv):
                if means[l, a] > means[l, b] + 1e-8:
                    assert caps[l, a] >= caps[l, b]
    layer_tot = caps.sum(axis=1)                             # and layer totals monotone in the layer's INF
    ls = means.sum(axis=1)
    for a in range(L):
        for b in range(L):
            if ls[a] > ls[b] + 1e-7:
                assert layer_tot[a] >= layer_tot[b]


def test_exact_single_layer_is_proportional():
    inf = [[0.8, 0.1, 0.1, 0.0]]
    caps = oracle.allocate_budgets(inf, 4, 4, 260, 10)
    assert caps == [[10 + 800, 10 + 100, 10 + 100, 10]]


def test_exact_scale_invariance_and_permutation():
    rng = np.random.default_rng(3)
    grid = rng.integers(1, 2 ** 10, size=(3, 4)) / 2.0 ** 12        # exact on the fixed-point grid
    a = oracle.allocate_budgets(grid.tolist(), 4, 4, 77, 7)
    b = oracle.allocate_budgets((grid * 4).tolist(), 4, 4, 77, 7)
    assert a == b
    perm = [2, 0, 3, 1]
    c = oracle.allocate_budgets(grid[:, perm].tolist(), 4, 4, 77, 7)
    assert sorted(map(sorted, c)) == sorted(map(sorted, a)) or np.abs(
        np.sort(np.array(c), axis=1) - np.sort(np.array(a), axis=1)).max() <= 1


def test_layer_floor_share():
    # a layer with zero INF still receives 0.01/(1 + 0.01 L) of the pool (the minimum layer share)
    inf = [[0.5, 0.5], [0.0, 0.0]]
    caps = np.array(oracle.allocate_budgets(inf, 2, 2, 1000, 0))
    pool = 1000 * 4
    share = Fraction(1, 100) / (1 + Fraction(2, 100))
    assert abs(int(caps[1].sum()) - float(pool * share)) < 1.0
    assert caps[1, 0] - caps[1, 1] in (0, 1)


def test_rejects_bad_inputs():
    with pytest.raises(ValueError):
        oracle.allocate_budgets([[1.5]], 1, 1, 10, 2)
    with pytest.raises(ValueError):
        oracle.allocate_budgets([[0.5]], 1, 1, 10, 12)
    with pytest.raises(ValueError):
        oracle.allocate_budgets([[0.5, 0.1, 0.2]], 3, 2, 10, 2)
