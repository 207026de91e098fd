"""GPU parity of slkv_score_heads against the float64 oracle, through the C ABI.

The four weight cells are sums of fp32 inputs taken in float64 on both sides, so they agree to
rounding order: relative 1e-12 (absolute 1e-15 for cells that are zero in exact arithmetic)."""

import numpy as np
import pytest

import oracle
from paper_2508_15806_amd import api
from paper_2508_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run(rows, start, length, topk, acc=None):
    import torch
    d_rows = torch.from_numpy(np.ascontiguousarray(rows)).cuda()
    d_acc = None if acc is None else torch.from_numpy(acc.copy()).cuda()
    acc_d, sc_d = api.score_heads(d_rows, start, length, topk, d_acc)
    torch.cuda.synchronize()
    return acc_d.cpu().numpy(), sc_d.cpu().numpy()


def check(rows, start, length, topk):
    acc, scores = run(rows, start, length, topk)
    racc, rscores = oracle.score_heads(rows, start, length, topk)
    np.testing.assert_allclose(acc, racc, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(scores, rscores, rtol=1e-11, atol=1e-15)
    return acc, scores


def test_config4_shape_rows_resident():
    nr = wl.config4(L=2, H=4, T=16, n=16384)
    acc, scores = check(nr.rows, nr.needle_start, nr.needle_len, nr.topk)
    assert (acc[..., 4] == 16).all()
    np.testing.assert_allclose(acc[..., :4].sum(-1), 16.0, rtol=1e-6)


@pytest.mark.parametrize("n,topk", [(4, 1), (8, 8), (64, 1), (1000, 32), (5003, 100), (4096, 4096), (4096, 65), (16384, 64),
                                    (16388, 64), (20000, 17), (70001, 64)])
def test_row_lengths_and_k(n, topk):
    nr = wl.config4(L=1, H=3, T=5, n=n, needle_len=max(1, min(32, n // 2)), seed_extra=n)
    check(nr.rows, nr.needle_start, nr.needle_len, topk)


def test_ties_are_cut_by_lowest_position():
    # uniform rows: T_k = [0, K); closed forms for a needle at the start, and nothing for one after K
    n, K = 4096, 32
    rows = np.full((1, 2, 3, n), 1.0 / n, dtype=np.float32)
    acc, scores = check(rows, 0, 16, K)
    np.testing.assert_allclose(scores[0, 0], [16 / 32, 1.0, 2 * 0.5 / 1.5], rtol=1e-12)
    acc, scores = check(rows, K, 16, K)
    assert (scores == 0).all()
    acc, scores = check(rows, 20, 24, K)                       # needle straddles the cut
    np.testing.assert_allclose(scores[0, 0, :2], [12 / 32, 12 / 24], rtol=1e-12)
    # quantised weights: many ties at the K-th value, non-resident and resident lengths
    rng = np.random.default_rng(3)
    for n in (3001, 8192):
        q = rng.integers(0, 6, size=(2, 2, 4, n)).astype(np.float32)
        q /= q.sum(-1, keepdims=True)
        for start, K in ((0, 50), (n // 2, 700), (n - 40, 40)):
            check(q.astype(np.float32), start, 40, K)


def test_accumulates_across_calls():
    a = wl.config4(L=2, H=2, T=4, n=2048, seed_extra=1)
    b = wl.config4(L=2, H=2, T=4, n=4096, seed_extra=2)
    acc1, _ = run(a.rows, a.needle_start, a.needle_len, a.topk)
    acc2, sc2 = run(b.rows, b.needle_start, b.needle_len, b.topk, acc=acc1)
    r1, _ = oracle.score_heads(a.rows, a.needle_start, a.needle_len, a.topk)
    r2, rs2 = oracle.score_heads(b.rows, b.needle_start, b.needle_len, b.topk, acc=r1)
    np.testing.assert_allclose(acc2, r2, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(sc2, rs2, rtol=1e-11, atol=1e-15)


def test_two_runs_are_bit_identical():
    nr = wl.config4(L=2, H=2, T=8, n=16384, seed_extra=9)
    a = run(nr.rows, nr.needle_start, nr.needle_len, nr.topk)
    b = run(nr.rows, nr.needle_start, nr.needle_len, nr.topk)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_config4_full_launch_shape_sampled_heads():
    # the benchmark's launch configuration (32 x 32 heads x 16 rows of 16384 weights = 1 GiB, one
    # workgroup per row); 8 generated layers are repeated four times on the device, and a sample
    # of heads is checked against the oracle
    import torch
    nr = wl.config4(L=8)
    d_rows = torch.from_numpy(nr.rows).cuda().repeat(4, 1, 1, 1)
    assert tuple(d_rows.shape) == (32, 32, 16, 16384)
    acc_d, sc_d = api.score_heads(d_rows, nr.needle_start, nr.needle_len, nr.topk)
    torch.cuda.synchronize()
    acc, scores = acc_d.cpu().numpy(), sc_d.cpu().numpy()
    rng = np.random.default_rng(5)
    picks = {(int(l), int(h)) for l, h in zip(rng.integers(0, 32, 40), rng.integers(0, 32, 40))}
    # heads whose rows touch the needle are the interesting ones: add those with the largest WO
    top = np.argsort(acc[..., 0].ravel())[-8:]
    picks |= {(int(i // 32), int(i % 32)) for i in top}
    for l, h in sorted(picks):
        racc, rsc = oracle.score_heads(nr.rows[l % 8:l % 8 + 1, h:h + 1], nr.needle_start, nr.needle_len, nr.topk)
        np.testing.assert_allclose(acc[l, h], racc[0, 0], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(scores[l, h], rsc[0, 0], rtol=1e-11, atol=1e-15)
    assert (acc[..., 4] == 16).all()


@pytest.mark.parametrize("agg,comps", [("micro", (True, True, True)), ("macro", (True, True, True)),
                                       ("micro", (True, True, False)), ("micro", (True, False, True)),
                                       ("macro", (True, False, True)), ("micro", (False, True, True)),
                                       ("macro", (True, False, False))])
def test_aggregation_and_ablation_modes(agg, comps):
    import torch
    from paper_2508_15806_amd import api, binding as B
    nr = wl.config4(L=2, H=5, T=7, n=4096, seed_extra=11)
    rows = torch.from_numpy(nr.rows).cuda()
    mode = B.SLKV_AGG_MACRO if agg == "macro" else B.SLKV_AGG_MICRO
    acc, sc = api.score_heads_ex(rows, nr.needle_start, nr.needle_len, nr.topk, mode, comps)
    acc, sc = api.score_heads_ex(rows, nr.needle_start, nr.needle_len, nr.topk, mode, comps, acc=acc)   # accumulates
    torch.cuda.synchronize()
    racc, rsc = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk, agg, comps)
    racc, rsc = oracle.score_heads_modes(nr.rows, nr.needle_start, nr.needle_len, nr.topk, agg, comps, acc=racc)
    np.testing.assert_allclose(acc.cpu().numpy(), racc, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(sc.cpu().numpy(), rsc, rtol=1e-11, atol=1e-15)
