"""GPU parity of slkv_score_heads_qk (Stage 1 straight from decode queries and context keys, the
attention rows never in memory) against the float64 oracle, through the C ABI.

The GPU computes logits as fp32 sums of exact bf16 products and weights as fp32 exponentials, the
oracle everything in float64: weights agree to about 1e-5 relative, so do the cells (sums of at
most K weights per row).  Two logits closer than fp32 rounding could rank differently on the two
sides; the seeded inputs here hold no such pair at the K-th place (a flip would move a whole
weight between cells and fail the comparison)."""

import numpy as np
import pytest

import oracle
from paper_2508_15806_amd import api
from paper_2508_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu

RTOL, ATOL = 2e-4, 2e-7


def run_gpu(x, acc=None):
    import torch
    q = api.to_device(x.q, "bf16")
    k = api.to_device(x.k, "bf16")
    acc_d, sc_d = api.score_heads_qk(q, k, x.needle_start, x.needle_len, x.topk, acc)
    torch.cuda.synchronize()
    return acc_d, sc_d


def check(x):
    acc_d, sc_d = run_gpu(x)
    racc, rsc = oracle.score_heads_from_qk(x.q, x.k, x.needle_start, x.needle_len, x.topk)
    np.testing.assert_allclose(acc_d.cpu().numpy(), racc, rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(sc_d.cpu().numpy(), rsc, rtol=5 * RTOL, atol=1e-6)
    return acc_d, racc


def test_one_row_group_ragged_context():
    # 64 rows per KV head (4 query heads x 16 steps); n is no multiple of the 32-key sub-tile or of a stripe of them
    check(wl.config4_qk(L=2, Hq=8, Hkv=2, T=16, n=4096 + 37, d=128))


def test_partial_row_group_head_dim_64_small_k():
    x = wl.config4_qk(L=1, Hq=8, Hkv=2, T=5, n=700, d=64, needle_len=5, seed_extra=1)
    x.topk = 8
    check(x)


@pytest.mark.parametrize("n,topk,d", [(40, 8, 128), (257, 16, 64), (1024, 64, 128), (1025, 1, 128), (5000, 64, 128)])
def test_short_contexts_and_the_largest_k(n, topk, d):
    # fewer keys than one stripe of sub-tiles, exactly the first chunk, one key more, K = 1 and the largest K
    x = wl.config4_qk(L=1, Hq=4, Hkv=2, T=7, n=n, d=d, needle_len=min(16, n // 2), seed_extra=10 + n)
    x.topk = topk
    check(x)


def test_several_row_groups_and_accumulation():
    import torch
    x = wl.config4_qk(L=1, Hq=8, Hkv=1, T=12, n=3000, d=128, seed_extra=2)      # 96 rows per KV head: 64 + 32
    acc_d, racc = check(x)
    acc_d, _ = run_gpu(x, acc_d)                                                 # a second call adds to the accumulators
    np.testing.assert_allclose(acc_d.cpu().numpy(), 2 * racc, rtol=RTOL, atol=ATOL)


def test_rows_of_equal_logits_go_through_the_fallback():
    # identical keys under the first KV head: every logit of its rows ties, T_k is the K lowest positions
    x = wl.config4_qk(L=1, Hq=4, Hkv=2, T=3, n=1500, d=128, needle_len=16, seed_extra=3, tie_rows=1)
    x.needle_start, x.topk = 8, 16                                                # needle [8, 24) against T_k = [0, 16)
    acc_d, racc = check(x)
    got = acc_d.cpu().numpy()
    np.testing.assert_allclose(got[0, 0, :3], [3 * 8 / 1500, 3 * 8 / 1500, 3 * 8 / 1500], rtol=1e-6)


def test_logits_rising_along_the_context_overflow_into_the_fallback():
    # keys of the first KV head = (j / n) * v: rows with q.v > 0 see logits that rise with the position, so every
    # chunk of keys beats the bound taken from the chunks before it and the candidate lists overflow; rows with
    # q.v < 0 have their top-K at the very beginning
    x = wl.config4_qk(L=1, Hq=8, Hkv=2, T=8, n=6000 + 13, d=128, needle_len=16, seed_extra=4)
    n = x.k.shape[2]
    v = np.random.default_rng(9).standard_normal(128).astype(np.float32)
    ramp = (np.arange(n, dtype=np.float32) / n * 6.0)[:, None] * v[None, :]
    x.k[0, 0] = wl.to_bf16_bits(ramp)
    x.needle_start = n - 40
    check(x)


def test_needle_run_shape_sampled_heads():
    # the shape bench.py times (32 layers x 32 query / 8 KV heads, 16 steps, 16384 keys); the oracle takes sampled heads
    x = wl.config4_qk()
    acc_d, sc_d = run_gpu(x)
    got_acc, got_sc = acc_d.cpu().numpy(), sc_d.cpu().numpy()
    rng = np.random.default_rng(0)
    for l, kv in zip(rng.integers(0, 32, size=6).tolist(), rng.integers(0, 8, size=6).tolist()):
        racc, rsc = oracle.score_heads_from_qk(x.q[l:l + 1, kv * 4:kv * 4 + 4], x.k[l:l + 1, kv:kv + 1], x.needle_start,
                                               x.needle_len, x.topk)
        np.testing.assert_allclose(got_acc[l, kv * 4:kv * 4 + 4], racc[0], rtol=RTOL, atol=ATOL)
        np.testing.assert_allclose(got_sc[l, kv * 4:kv * 4 + 4], rsc[0], rtol=5 * RTOL, atol=1e-6)
    # every row's cells sum to one row of mass
    np.testing.assert_allclose(got_acc[..., :4].sum(axis=-1), 16.0, rtol=1e-6)
