"""Pins for oracle/compress.py (CPU only).

Each test checks the oracle against something other than itself: brute-force
Python loops with un-stabilised exponentials, scipy routines, closed forms and
the structural facts Algorithm 3 fixes.  A dropped term, a wrong sign or axis,
a transposed operand or a wrong tie rule fails at least one of them."""

import math

import numpy as np
import pytest
import scipy.ndimage
import scipy.special

import oracle
from oracle import compress as oc
from paper_2508_15806_amd import workloads as wl


def brute_importance(q, k):
    """Eq. (2)-(4) with explicit loops and no max-subtraction."""
    G, w, d = q.shape
    m = k.shape[0]
    out = [0.0] * m
    for g in range(G):
        for i in range(w):
            logits = []
            for j in range(m):
                acc = 0.0
                for p in range(d):
                    acc += float(q[g, i, p]) * float(k[j, p])
                logits.append(acc / math.sqrt(d))
            ex = [math.exp(s) for s in logits]
            z = sum(ex)
            for j in range(m):
                out[j] += ex[j] / z
    return np.array(out)


def test_importance_matches_brute_force():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((2, 3, 8)).astype(np.float32)
    k = rng.standard_normal((17, 8)).astype(np.float32)
    got = oracle.window_importance(q, k)
    np.testing.assert_allclose(got, brute_importance(q, k), rtol=1e-12, atol=0)


def test_importance_matches_scipy_softmax_and_is_not_transposed():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((4, 5, 16)).astype(np.float32)
    k = rng.standard_normal((33, 16)).astype(np.float32)
    s = np.einsum("gwd,md->gwm", q.astype(np.float64), k.astype(np.float64)) / 4.0
    ref = scipy.special.softmax(s, axis=-1).sum(axis=(0, 1))
    np.testing.assert_allclose(oracle.window_importance(q, k), ref, rtol=1e-12)
    # softmax over the wrong axis would not give row sums of one
    assert abs(ref.sum() - 20.0) < 1e-9


def test_importance_sum_is_rows():
    lay = wl.make_layer((7, 7), [300], 8, 2, 64, 16, dtype="bf16", bias_frac=0.05)
    imp = oracle.window_importance(lay.qwin[0, 0:4], lay.k[0, :284])
    assert abs(imp.sum() - 4 * 16) < 1e-10
    assert (imp > 0).all()


def test_zero_queries_give_uniform_importance():
    q = np.zeros((2, 4, 8), dtype=np.float32)
    k = np.random.default_rng(3).standard_normal((50, 8)).astype(np.float32)
    imp = oracle.window_importance(q, k)
    np.testing.assert_allclose(imp, np.full(50, 8 / 50), rtol=1e-14)


def test_planted_key_takes_all_mass():
    rng = np.random.default_rng(4)
    q = rng.standard_normal((1, 4, 16)).astype(np.float32)
    k = rng.standard_normal((40, 16)).astype(np.float32) * 0.01
    # a key aligned with the mean query direction, very long
    k[13] = 400.0 * np.sign(q[0].sum(axis=0))
    q = np.abs(q) * np.sign(q[0].sum(axis=0))       # every query agrees in sign with k[13]
    imp = oracle.window_importance(q.astype(np.float32), k)
    assert imp.argmax() == 13
    assert abs(imp[13] - 4.0) < 1e-9


def test_scale_is_inverse_sqrt_d():
    # one query, two keys: softmax of (a, 0)/sqrt(d) has closed form 1/(1+exp(-a/sqrt(d)))
    d = 64
    q = np.zeros((1, 1, d), dtype=np.float32)
    q[0, 0, 0] = 8.0
    k = np.zeros((2, d), dtype=np.float32)
    k[0, 0] = 2.0
    imp = oracle.window_importance(q, k)
    assert abs(imp[0] - 1.0 / (1.0 + math.exp(-16.0 / 8.0))) < 1e-14


def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x3DCD], dtype=np.uint16)
    vals = oracle.bf16_bits_to_f64(bits)
    assert vals[0] == 1.0 and vals[1] == -1.0 and vals[3] == 0.0
    assert vals[2] == 3.140625
    assert vals[4] == float(np.array([0x3DCD0000], dtype=np.uint32).view(np.float32)[0])
    # round trip through the generator's rounding
    x = np.random.default_rng(5).standard_normal(1000).astype(np.float32)
    b = wl.to_bf16_bits(x)
    assert np.all(np.abs(oracle.bf16_bits_to_f64(b) - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(wl.to_bf16_bits(wl.bf16_bits_to_f32(b)), b)


def test_fp16_widening_is_exact_and_the_layer_equals_its_fp32_copy():
    h = np.array([1.0, -1.0, 3.140625, 0.0, 6.103515625e-05, 65504.0], dtype=np.float16)
    assert oracle.bf16_bits_to_f64(h).tolist() == [1.0, -1.0, 3.140625, 0.0, 2.0 ** -14, 65504.0]
    # a half-precision layer and the same values stored as fp32 are the same problem
    lay = wl.make_layer((41,), [300, 77], 4, 2, 64, 16, dtype="f16", bias_frac=0.05)
    bud = np.array([60, 100], dtype=np.int32)
    a = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, bud, lay.w, 7)
    b = oracle.compress_layer(lay.qwin.astype(np.float32), lay.k.astype(np.float32), lay.v.astype(np.float32),
                              lay.cu_seqlens, bud, lay.w, 7)
    for sa, sb in zip(a["segments"], b["segments"]):
        assert np.array_equal(sa["kept_idx"], sb["kept_idx"]) and np.array_equal(sa["importance"], sb["importance"])
    assert a["k_out"].dtype == np.float16 and np.array_equal(a["k_out"].astype(np.float32), b["k_out"])


def test_e4m3_widening_follows_the_format_and_the_generator_rounds_to_nearest_even():
    v = oracle.fp8_e4m3_to_f64(np.arange(256, dtype=np.uint8))
    # bias 7, three mantissa bits, subnormals m * 2^-9, largest finite value 448, S.1111.111 = NaN
    assert v[0x38] == 1.0 and v[0x39] == 1.125 and v[0x40] == 2.0 and v[0x7E] == 448.0 and v[0x08] == 2.0 ** -6
    assert v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9 and v[0x00] == 0.0 and v[0xB8] == -1.0
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF]) and np.isfinite(np.delete(v, [0x7F, 0xFF])).all()
    assert (np.diff(v[:0x7F]) > 0).all()                      # codes of one sign are ordered like their values
    x = np.array([1.0625, 1.1875, 2.0 ** -10, 1000.0, -0.3, 0.0], dtype=np.float32)
    assert wl.to_fp8_e4m3_bits(x).tolist() == [0x38, 0x3A, 0x00, 0x7E, 0xAA, 0x00]      # ties to even, saturation
    fin = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    assert np.array_equal(wl.to_fp8_e4m3_bits(v[fin].astype(np.float32)) & 0x7F, fin & 0x7F)
    # a layer with E4M3 keys / values is the same problem as its values stored in fp32
    lay = wl.make_layer((42,), [300, 77], 4, 2, 64, 16, dtype="bf16_kv8", bias_frac=0.05)
    bud = np.array([60, 100], dtype=np.int32)
    a = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, bud, lay.w, 7)
    b = oracle.compress_layer(oracle.bf16_bits_to_f64(lay.qwin).astype(np.float32), oracle.fp8_e4m3_to_f64(lay.k).astype(np.float32),
                              oracle.fp8_e4m3_to_f64(lay.v).astype(np.float32), lay.cu_seqlens, bud, lay.w, 7)
    for sa, sb in zip(a["segments"], b["segments"]):
        assert np.array_equal(sa["kept_idx"], sb["kept_idx"]) and np.array_equal(sa["importance"], sb["importance"])
    assert a["k_out"].dtype == np.uint8


@pytest.mark.parametrize("kernel", [1, 3, 7, 9])
def test_max_pool_matches_scipy_and_loop(kernel):
    x = np.random.default_rng(6).random(101)
    got = oracle.pool_1d(x, kernel, oc.POOL_MAX)
    ref = scipy.ndimage.maximum_filter1d(x, size=kernel, mode="constant", cval=-np.inf)
    np.testing.assert_array_equal(got, ref)
    r = kernel // 2
    loop = np.array([max(x[max(0, j - r):j + r + 1]) for j in range(101)])
    np.testing.assert_array_equal(got, loop)
    assert (got >= x).all()
    if kernel == 1:
        np.testing.assert_array_equal(got, x)


@pytest.mark.parametrize("kernel", [3, 7])
def test_avg_pool_matches_convolve(kernel):
    x = np.random.default_rng(7).random(64)
    got = oracle.pool_1d(x, kernel, oc.POOL_AVG)
    ref = np.convolve(x, np.ones(kernel) / kernel, mode="same")
    np.testing.assert_allclose(got, ref, rtol=1e-13)


def test_pool_shorter_than_kernel():
    x = np.array([0.1, 0.5, 0.2])
    np.testing.assert_array_equal(oracle.pool_1d(x, 7, oc.POOL_MAX), [0.5, 0.5, 0.5])


def brute_topk(scores, k):
    order = sorted(range(len(scores)), key=lambda j: (-scores[j], j))
    return sorted(order[:k])


def test_topk_matches_full_sort_with_ties():
    rng = np.random.default_rng(8)
    for trial in range(20):
        m = int(rng.integers(1, 60))
        scores = rng.integers(0, 6, size=m).astype(np.float64) / 7.0   # many ties
        k = int(rng.integers(0, m + 1))
        idx, tau = oracle.select_topk(scores, k)
        assert idx.tolist() == brute_topk(scores.tolist(), k)
        assert len(idx) == k
        if k:
            assert tau == sorted(scores.tolist(), reverse=True)[k - 1]
        else:
            assert tau is None


def test_topk_special_cases():
    const = np.full(10, 0.3)
    assert oracle.select_topk(const, 4)[0].tolist() == [0, 1, 2, 3]
    assert oracle.select_topk(const, 0)[0].tolist() == []
    assert oracle.select_topk(const, 10)[0].tolist() == list(range(10))
    # a plateau cut in the middle keeps its lowest positions
    s = np.array([0.1, 0.9, 0.5, 0.5, 0.5, 0.5, 0.2])
    assert oracle.select_topk(s, 3)[0].tolist() == [1, 2, 3]


def small_layer(dtype="bf16", seqlens=(90, 40), Hq=4, Hkv=2, d=16, w=8):
    return wl.make_layer((11, 3), list(seqlens), Hq, Hkv, d, w, dtype=dtype, bias_frac=0.1)


def test_segment_structure():
    lay = small_layer()
    w = lay.w
    res = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, [20, 50], w, 7)
    offs = res["out_offsets"]
    assert offs[0] == 0
    s = 0
    for b in range(lay.B):
        n = int(lay.cu_seqlens[b + 1] - lay.cu_seqlens[b])
        for h, cap in enumerate([20, 50]):
            seg = res["segments"][b * 2 + h]
            idx = seg["kept_idx"]
            assert len(idx) == oracle.kept_count(n, w, cap)
            assert offs[s + 1] - offs[s] == len(idx)
            if n <= cap:
                assert idx.tolist() == list(range(n))
                assert seg["pooled"] is None
            else:
                assert idx[-w:].tolist() == list(range(n - w, n))       # window kept, last, in order
                hist = idx[:-w]
                assert len(hist) == cap - w
                assert (np.diff(hist) > 0).all() and hist.max() < n - w
                assert hist.tolist() == brute_topk(seg["pooled"].tolist(), cap - w)
            # gather is a bit copy of the input rows
            t0 = int(lay.cu_seqlens[b])
            assert np.array_equal(seg["k_out"], lay.k[h, t0 + idx])
            assert np.array_equal(seg["v_out"], lay.v[h, t0 + idx])
            assert np.array_equal(res["k_out"][offs[s]:offs[s + 1]], seg["k_out"])
            assert seg["k_out"].dtype == lay.k.dtype
            s += 1
    assert offs[-1] == res["k_out"].shape[0] == res["v_out"].shape[0]


def test_short_sequence_is_returned_unchanged():
    lay = small_layer(seqlens=(30,))
    res = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, [30, 64], lay.w, 7)
    for h in range(2):
        assert np.array_equal(res["segments"][h]["k_out"], lay.k[h])
        assert np.array_equal(res["segments"][h]["v_out"], lay.v[h])


def test_capacity_below_window_keeps_window_only():
    lay = small_layer(seqlens=(64,))
    res = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, [3, 8], lay.w, 7)
    for h in range(2):
        assert res["segments"][h]["kept_idx"].tolist() == list(range(56, 64))


def test_gqa_uses_the_right_query_heads():
    # importance of KV head 1 must come from query heads 2,3 (G=2), not 0,1 or 1,2
    lay = small_layer(dtype="f32", seqlens=(70,))
    res = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, [20, 20], lay.w, 1)
    ref = brute_importance(lay.qwin[0, 2:4], lay.k[1, :62])
    np.testing.assert_allclose(res["segments"][1]["importance"], ref, rtol=1e-11)


def test_ragged_batch_uses_own_tokens():
    lay = small_layer(dtype="f32", seqlens=(50, 45))
    res = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, [20, 20], lay.w, 1)
    ref = brute_importance(lay.qwin[1, 0:2], lay.k[0, 50:50 + 37])
    np.testing.assert_allclose(res["segments"][2]["importance"], ref, rtol=1e-11)


def test_score_cache_is_memoisation_only():
    # the cached scores of one budget row reused under other budgets give what a fresh call gives
    lay = wl.make_layer((8, 1), [400, 120], 8, 2, 64, 16, dtype="bf16", bias_frac=0.05)
    cache = {}
    for bud in ([300, 40], [60, 17], [30, 399], [1000, 5]):
        a = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, bud, lay.w, 5, oc.POOL_MAX, score_cache=cache)
        b = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, bud, lay.w, 5, oc.POOL_MAX)
        assert np.array_equal(a["out_offsets"], b["out_offsets"])
        assert np.array_equal(a["k_out"], b["k_out"]) and np.array_equal(a["v_out"], b["v_out"])
        for sa, sb in zip(a["segments"], b["segments"]):
            assert np.array_equal(sa["kept_idx"], sb["kept_idx"]) and sa["tau"] == sb["tau"]
    assert set(cache) == {(0, 0), (0, 1), (1, 0), (1, 1)}
