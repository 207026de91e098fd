"""Pins of oracle.recompress_layer (Algorithm 3 on an already compacted cache, Section 3.4).

The per-segment arithmetic is compress_segment, pinned in test_oracle_compress.py; what is new
here is the ragged addressing and the position bookkeeping, pinned by an explicit loop
implementation on tiny inputs, by equivalence with the packed-batch layout when every head has
the same length, and by the invariants of a prefill -> decode -> re-compress chain."""

import math

import numpy as np

import oracle
from paper_2508_15806_amd import workloads as wl


def brute_segment(q_group, k_seg, v_seg, w, cap):
    """Direct loops: no pooling (kernel 1); returns kept positions."""
    n, d = k_seg.shape
    if n <= w or n <= cap:
        return list(range(n))
    m = n - w
    kk = min(max(cap - w, 0), m)
    score = [0.0] * m
    for g in range(q_group.shape[0]):
        for i in range(w):
            logits = [sum(float(q_group[g, i, p]) * float(k_seg[j, p]) for p in range(d)) / math.sqrt(d) for j in range(m)]
            mx = max(logits)
            e = [math.exp(x - mx) for x in logits]
            z = sum(e)
            for j in range(m):
                score[j] += e[j] / z
    order = sorted(range(m), key=lambda j: (-score[j], j))
    return sorted(order[:kk]) + list(range(m, n))


def test_matches_explicit_loops_on_a_tiny_ragged_cache():
    rc = wl.make_ragged_cache((901,), [9, 14, 5, 20, 3, 11], 3, 4, 2, 8, 3, dtype="f32", seq_len=64)
    budgets = [6, 9]
    ref = oracle.recompress_layer(rc.qwin, rc.k_rows, rc.v_rows, rc.in_offsets, budgets, rc.w, 1,
                                  oracle.compress.POOL_NONE, pos_in=rc.pos_in)
    G = 2
    run = 0
    for s in range(6):
        b, h = divmod(s, 2)
        r0, r1 = int(rc.in_offsets[s]), int(rc.in_offsets[s + 1])
        want = brute_segment(rc.qwin[b, h * G:(h + 1) * G], rc.k_rows[r0:r1], rc.v_rows[r0:r1], rc.w, budgets[h])
        got = ref["segments"][s]["kept_idx"].tolist()
        assert got == want, s
        assert ref["out_offsets"][s] == run
        assert np.array_equal(ref["k_out"][run:run + len(want)], rc.k_rows[r0 + np.array(want, dtype=np.int64)])
        assert np.array_equal(ref["v_out"][run:run + len(want)], rc.v_rows[r0 + np.array(want, dtype=np.int64)])
        assert np.array_equal(ref["pos_out"][run:run + len(want)], rc.pos_in[r0 + np.array(want, dtype=np.int64)])
        run += len(want)
    assert ref["out_offsets"][6] == run


def test_equal_head_lengths_reduce_to_the_packed_batch_layout():
    lay = wl.make_layer((902,), [150, 90], 4, 2, 64, 8, dtype="bf16", bias_frac=0.05)
    budgets = [40, 77]
    a = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, budgets, lay.w)
    # the same keys laid out segment after segment
    rows_k, rows_v, offs = [], [], [0]
    for b in range(2):
        t0, t1 = int(lay.cu_seqlens[b]), int(lay.cu_seqlens[b + 1])
        for h in range(2):
            rows_k.append(lay.k[h, t0:t1])
            rows_v.append(lay.v[h, t0:t1])
            offs.append(offs[-1] + t1 - t0)
    r = oracle.recompress_layer(lay.qwin, np.concatenate(rows_k), np.concatenate(rows_v), offs, budgets, lay.w)
    assert np.array_equal(a["out_offsets"], r["out_offsets"])
    assert np.array_equal(a["k_out"], r["k_out"]) and np.array_equal(a["v_out"], r["v_out"])
    for sa, sr in zip(a["segments"], r["segments"]):
        assert np.array_equal(sa["kept_idx"], sr["kept_idx"])


def test_prefill_then_decode_chain_invariants():
    w, budgets = 8, [30, 12, 100, 5]
    rc = wl.make_ragged_cache((903,), [60, 20, 90, 33], 1, 8, 4, 64, w, dtype="bf16", bias_frac=0.05, seq_len=500)
    r = oracle.recompress_layer(rc.qwin, rc.k_rows, rc.v_rows, rc.in_offsets, budgets, w, pos_in=rc.pos_in)
    for s, (n, cap) in enumerate(zip([60, 20, 90, 33], budgets)):
        o0, o1 = int(r["out_offsets"][s]), int(r["out_offsets"][s + 1])
        assert o1 - o0 == oracle.kept_count(n, w, cap) == (n if n <= cap else max(cap, w))
        p = r["pos_out"][o0:o1]
        assert (np.diff(p) > 0).all()                       # temporal order survives
        assert np.array_equal(p[-w:], np.arange(500 - w, 500))   # the newest w tokens are always kept
    # a cache within capacity comes back bit-identical
    big = [1000] * 4
    r2 = oracle.recompress_layer(rc.qwin, rc.k_rows, rc.v_rows, rc.in_offsets, big, w, pos_in=rc.pos_in)
    assert np.array_equal(r2["k_out"], rc.k_rows) and np.array_equal(r2["pos_out"], rc.pos_in)
    assert np.array_equal(r2["out_offsets"], rc.in_offsets)
    # compressing the compressed cache again with the same capacities keeps it whole (length == capacity)
    r3 = oracle.recompress_layer(rc.qwin, r["k_out"], r["v_out"], r["out_offsets"], budgets, w, pos_in=r["pos_out"])
    for s, cap in enumerate(budgets):
        o0, o1 = int(r["out_offsets"][s]), int(r["out_offsets"][s + 1])
        if o1 - o0 <= cap:
            q0, q1 = int(r3["out_offsets"][s]), int(r3["out_offsets"][s + 1])
            assert np.array_equal(r3["pos_out"][q0:q1], r["pos_out"][o0:o1])
