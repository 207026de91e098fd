"""Pins for oracle.attention_rows / score_heads_from_qk (CPU only): explicit loops with
un-stabilised exponentials, the grouped-query head mapping, and Algorithm 1 by brute force on the rows."""

import math

import numpy as np

import oracle
from paper_2508_15806_amd import workloads as wl


def brute_row(qv, keys):
    d = len(qv)
    logits = [sum(float(qv[p]) * float(kr[p]) for p in range(d)) / math.sqrt(d) for kr in keys]
    ex = [math.exp(s) for s in logits]
    z = sum(ex)
    return [e / z for e in ex]


def test_rows_match_explicit_loops_and_use_the_group_s_kv_head():
    rng = np.random.default_rng(5)
    q = rng.standard_normal((2, 4, 3, 8)).astype(np.float32)
    k = rng.standard_normal((2, 2, 11, 8)).astype(np.float32)
    rows = oracle.attention_rows(q, k)
    assert rows.shape == (2, 4, 3, 11)
    for l in range(2):
        for h in range(4):
            for t in range(3):
                np.testing.assert_allclose(rows[l, h, t], brute_row(q[l, h, t], k[l, h // 2]), rtol=1e-12)
    np.testing.assert_allclose(rows.sum(axis=-1), 1.0, rtol=1e-14)
    # heads 0,1 share KV head 0: swapping KV heads must change them
    rows2 = oracle.attention_rows(q, k[:, ::-1])
    assert not np.allclose(rows2[:, 0], rows[:, 0])


def test_bf16_inputs_are_widened_exactly():
    x = wl.config4_qk(L=1, Hq=4, Hkv=2, T=2, n=64, d=64)
    rows = oracle.attention_rows(x.q, x.k)
    qf, kf = wl.bf16_bits_to_f32(x.q), wl.bf16_bits_to_f32(x.k)
    np.testing.assert_allclose(rows[0, 3, 1], brute_row(qf[0, 3, 1], kf[0, 1]), rtol=1e-12)


def test_scores_from_qk_are_algorithm_1_on_those_rows():
    x = wl.config4_qk(L=1, Hq=4, Hkv=2, T=3, n=200, d=64, needle_len=8)
    acc, sc = oracle.score_heads_from_qk(x.q, x.k, x.needle_start, x.needle_len, x.topk)
    qf, kf = wl.bf16_bits_to_f32(x.q), wl.bf16_bits_to_f32(x.k)
    needle = set(range(x.needle_start, x.needle_start + x.needle_len))
    for h in range(4):
        WO = WD = WS = 0.0
        for t in range(3):
            row = brute_row(qf[0, h, t], kf[0, h // 2])
            top = sorted(range(200), key=lambda j: (-row[j], j))[:x.topk]
            wo = sum(row[j] for j in top if j in needle)
            WO += wo
            WD += sum(row[j] for j in top if j not in needle)
            WS += max(0.0, sum(row[j] for j in needle) - wo)
        np.testing.assert_allclose(acc[0, h, :3], [WO, WD, WS], rtol=1e-11, atol=1e-15)
        SF = WO / (WO + WD) if WO + WD > 0 else 0.0
        LG = WO / (WO + WS) if WO + WS > 0 else 0.0
        np.testing.assert_allclose(sc[0, h], [SF, LG, 2 * SF * LG / (SF + LG) if SF + LG > 0 else 0.0], rtol=1e-11)
