"""CPU-only tests of the C-ABI library's host side: it loads, exports every symbol the header
declares, allocates budgets exactly as the oracle does, and rejects bad arguments before any
GPU call."""

import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2508_15806_amd import binding as B
from paper_2508_15806_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "slkv.h")).read()
    declared = set(re.findall(r"\b(slkv_[a-z_0-9]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert B.slkv_version() == 1005
    assert L.slkv_status_str(0) == b"ok"


def test_desc_layout_matches_header():
    # 10 x 4 bytes, pointer, 4 x 8 bytes, pointer
    assert C.sizeof(B.LayerDesc) == 40 + 8 + 32 + 8


@pytest.mark.parametrize("seed", range(8))
def test_budgets_match_oracle_exact(seed):
    rng = np.random.default_rng(seed)
    L, Hkv, G = int(rng.integers(1, 33)), int(rng.integers(1, 9)), int(rng.choice([1, 2, 4, 8]))
    Hq = Hkv * G
    inf = [rng.random((L, Hq)), wl.inf_spiky((seed, 1), L, Hq), wl.inf_beta((seed, 2), L, Hq)][seed % 3]
    avg = int(rng.integers(1, 2000))
    fixed = int(rng.integers(0, avg + 1))
    got = B.slkv_allocate_budgets(inf, Hkv, avg, fixed)
    assert got.tolist() == oracle.allocate_budgets(inf.tolist(), Hq, Hkv, avg, fixed)
    assert int(got.sum()) == avg * L * Hkv
    lit = B.slkv_allocate_budgets(inf, Hkv, avg, fixed, B.SLKV_BUDGET_PAPER_LITERAL)
    assert lit.tolist() == oracle.allocate_budgets_literal(inf.tolist(), Hq, Hkv, avg, fixed)


def test_budgets_config3_map():
    inf = wl.config3_inf()
    for avg in wl.C3_BUDGETS:
        got = B.slkv_allocate_budgets(inf, 8, avg, 16)
        assert got.tolist() == oracle.allocate_budgets(inf.tolist(), 32, 8, avg, 16)
        assert int(got.sum()) == avg * 32 * 8 and int(got.min()) >= 16
    zero = B.slkv_allocate_budgets(np.zeros((3, 4)), 2, 10, 2)
    assert (zero == 10).all()


def test_fixed_from_beta():
    for avg, beta in [(64, 1.351), (128, 1.351), (128, 4 / 3), (512, 8 / 7), (1024, 1.0)]:
        assert B.slkv_fixed_from_beta(avg, beta) == oracle.fixed_from_beta(avg, beta)


def test_budget_errors():
    with pytest.raises(B.SlkvError) as e:
        B.slkv_allocate_budgets(np.array([[0.5, 1.5]]), 2, 10, 2)
    assert e.value.status == 3
    with pytest.raises(B.SlkvError) as e:
        B.slkv_allocate_budgets(np.array([[0.5, np.nan]]), 2, 10, 2)
    assert e.value.status == 3
    with pytest.raises(B.SlkvError) as e:
        B.slkv_allocate_budgets(np.array([[0.5, 0.5]]), 2, 10, 12)
    assert e.value.status == 2
    with pytest.raises(B.SlkvError) as e:
        B.slkv_allocate_budgets(np.array([[0.5, 0.5, 0.5]]), 2, 10, 2)
    assert e.value.status == 2
    assert B.lib().slkv_allocate_budgets(None, 1, 1, 1, 1, 0, 0, None) == 1


def make_layer(**over):
    args = dict(dtype=B.SLKV_BF16, B=2, Hq=8, Hkv=2, d=128, w=16, cu_seqlens=[0, 100, 130], budgets=[40, 120],
                k_strides=(128, 130 * 128), v_strides=(128, 130 * 128))
    args.update(over)
    return B.Layer(args["dtype"], args["B"], args["Hq"], args["Hkv"], args["d"], args["w"], args["cu_seqlens"],
                   args["budgets"], args["k_strides"], args["v_strides"], args.get("pool_kernel", 7),
                   args.get("pool", B.SLKV_POOL_MAX))


def test_compacted_sizes_follow_algorithm3():
    lay = make_layer()
    offs, total = B.slkv_compacted_sizes(lay)
    # seq 0 (n=100): cap 40 -> 40 rows; cap 120 -> all 100.  seq 1 (n=30): both keep all 30.
    assert offs.tolist() == [0, 40, 140, 170, 200] and total == 200
    lay = make_layer(budgets=[3, 16])
    offs, total = B.slkv_compacted_sizes(lay)       # capacity below the window: the window is kept
    assert offs.tolist() == [0, 16, 32, 48, 64]
    for n, w, cap in [(10, 16, 4), (100, 16, 40), (100, 16, 100), (100, 16, 8), (17, 16, 16)]:
        lay = make_layer(B=1, cu_seqlens=[0, n], budgets=[cap, cap], w=w, k_strides=(128, n * 128), v_strides=(128, n * 128))
        assert B.slkv_compacted_sizes(lay)[1] == 2 * oracle.kept_count(n, w, cap)
    assert B.slkv_workspace_bytes(make_layer()) > 0


@pytest.mark.parametrize("over,status", [
    (dict(d=96), 4), (dict(w=0), 2), (dict(pool_kernel=4), 2), (dict(pool_kernel=65), 2), (dict(pool=9), 2),
    (dict(Hq=7), 2), (dict(cu_seqlens=[0, 100, 90]), 2), (dict(budgets=[-1, 5]), 2), (dict(dtype=5), 2),
    (dict(k_strides=(64, 130 * 128)), 2), (dict(k_strides=(129, 130 * 128)), 2), (dict(Hq=128, w=64), 4),
    (dict(cu_seqlens=[0, 100, 2 ** 31]), 2),
])
def test_descriptor_validation(over, status):
    lay = make_layer(**over)
    with pytest.raises(B.SlkvError) as e:
        B.slkv_compacted_sizes(lay)
    assert e.value.status == status
    assert B.lib().slkv_last_error() != b""


def test_compress_rejects_before_touching_the_gpu():
    lay = make_layer()
    L = B.lib()
    args = [C.byref(lay.desc)] + [C.c_void_p(0)] * 9 + [C.c_int64(10), C.c_void_p(0), C.c_size_t(0), C.c_void_p(0)]
    assert L.slkv_compress_layer(*args) == 1                        # NULL pointers
    fake = C.c_void_p(4096)
    args = [C.byref(lay.desc)] + [fake] * 6 + [C.c_void_p(0)] * 3 + [C.c_int64(10), fake, C.c_size_t(0), C.c_void_p(0)]
    assert L.slkv_compress_layer(*args) == 5                        # workspace too small
    big = C.c_size_t(1 << 40)
    args = [C.byref(lay.desc)] + [fake] * 6 + [C.c_void_p(0)] * 3 + [C.c_int64(10), fake, big, C.c_void_p(0)]
    assert L.slkv_compress_layer(*args) == 6                        # output capacity too small
    odd = C.c_void_p(4100)
    args = [C.byref(lay.desc), odd] + [fake] * 5 + [C.c_void_p(0)] * 3 + [C.c_int64(1000), fake, big, C.c_void_p(0)]
    assert L.slkv_compress_layer(*args) == 2                        # misaligned pointer
    bad = B.LayerDesc()
    assert L.slkv_compress_layer(C.byref(bad), *args[1:]) == 2      # struct_size


def test_score_heads_validation():
    L = B.lib()
    fake = C.c_void_p(4096)
    big = C.c_size_t(1 << 40)
    null = C.c_void_p(0)
    ok = [fake, 2, 2, 2, C.c_int64(64), C.c_int64(8), 4, 4, fake, null, fake, big, null]

    def call(**kw):
        a = list(ok)
        for idx, val in kw.items():
            a[int(idx[1:])] = val
        return L.slkv_score_heads(*a)

    assert call(a0=null) == 1
    assert call(a4=C.c_int64(0)) == 2
    assert call(a5=C.c_int64(62)) == 2                               # needle runs past the row
    assert call(a7=0) == 2 and call(a7=65) == 2                      # topk outside 1..n
    assert call(a11=C.c_size_t(8)) == 5
    assert call(a0=C.c_void_p(4100)) == 2
    assert B.slkv_score_heads_workspace_bytes(2, 2, 2, 64) == 2 * 2 * 2 * 4 * 8


def make_ragged(**over):
    p = dict(dtype=B.SLKV_BF16, B=2, Hq=4, Hkv=2, d=128, w=16, in_offsets=[0, 100, 130, 130, 190], budgets=[40, 120],
             pool_kernel=7, pool=B.SLKV_POOL_MAX)
    p.update(over)
    return B.Ragged(p["dtype"], p["B"], p["Hq"], p["Hkv"], p["d"], p["w"], p["in_offsets"], p["budgets"],
                    p["pool_kernel"], p["pool"])


def test_recompress_sizes_follow_algorithm3():
    rag = make_ragged()
    offs, total = B.slkv_recompress_sizes(rag)
    # lengths 100, 30, 0, 60 with capacities 40, 120, 40, 120: 40 kept, all 30, nothing, all 60
    assert offs.tolist() == [0, 40, 70, 70, 130] and total == 130
    lens = [5, 17, 300, 64, 16, 1000]
    caps = [3, 100]
    rag = make_ragged(B=3, in_offsets=np.concatenate([[0], np.cumsum(lens)]), budgets=caps)
    offs, total = B.slkv_recompress_sizes(rag)
    want = [oracle.kept_count(n, 16, caps[i % 2]) for i, n in enumerate(lens)]
    assert np.diff(offs).tolist() == want and total == sum(want)
    assert B.slkv_recompress_workspace_bytes(rag) > 0


@pytest.mark.parametrize("over,status", [
    (dict(d=96), 4), (dict(w=0), 2), (dict(pool_kernel=4), 2), (dict(Hq=7), 2), (dict(budgets=[-1, 5]), 2),
    (dict(in_offsets=[0, 100, 90, 130, 190]), 2), (dict(in_offsets=[-1, 100, 130, 130, 190]), 2),
    (dict(in_offsets=[0, 100, 130, 130, 2 ** 31]), 2), (dict(dtype=7), 2),
])
def test_ragged_descriptor_validation(over, status):
    rag = make_ragged(**over)
    with pytest.raises(B.SlkvError) as e:
        B.slkv_recompress_sizes(rag)
    assert e.value.status == status


def test_recompress_rejects_before_touching_the_gpu():
    rag = make_ragged()
    L = B.lib()
    null, fake, odd = C.c_void_p(0), C.c_void_p(4096), C.c_void_p(4100)
    big = C.c_size_t(1 << 40)

    def call(q, kin, vin, pin, ko, vo, idx, po, cap, ws, wsb):
        return L.slkv_recompress_layer(C.byref(rag.desc), q, kin, vin, pin, ko, vo, idx, po, null, null, null,
                                       C.c_int64(cap), ws, wsb, null)
    assert call(null, null, null, null, null, null, null, null, 10, null, C.c_size_t(0)) == 1   # NULL pointers
    assert call(fake, fake, fake, fake, fake, fake, fake, null, 1000, fake, big) == 1           # pos_in without pos_out
    assert call(fake, fake, fake, null, fake, fake, fake, null, 1000, fake, C.c_size_t(0)) == 5  # workspace too small
    assert call(fake, fake, fake, null, fake, fake, fake, null, 10, fake, big) == 6             # output capacity
    assert call(odd, fake, fake, null, fake, fake, fake, null, 1000, fake, big) == 2            # misaligned pointer
    bad = B.RaggedDesc()
    assert L.slkv_recompress_layer(C.byref(bad), fake, fake, fake, null, fake, fake, fake, null, null, null, null,
                                   C.c_int64(1000), fake, big, null) == 2                       # struct_size


@pytest.mark.parametrize("seed", range(6))
def test_budgets_per_query_head_match_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    L, Hkv, G = int(rng.integers(1, 33)), int(rng.integers(1, 9)), int(rng.choice([1, 2, 4, 8]))
    Hq = Hkv * G
    inf = [rng.random((L, Hq)), wl.inf_spiky((seed, 3), L, Hq), wl.inf_beta((seed, 4), L, Hq)][seed % 3]
    avg, fixed = int(rng.integers(1, 2000)), 0
    fixed = int(rng.integers(0, avg + 1))
    got = B.slkv_allocate_budgets(inf, Hkv, avg, fixed, B.SLKV_BUDGET_EXACT_PER_QUERY_HEAD)
    assert got.tolist() == oracle.allocate_budgets_per_query_head(np.asarray(inf).tolist(), Hq, Hkv, avg, fixed)
    assert int(got.sum()) == avg * L * Hq


def test_score_heads_ex_rejects_bad_params_before_any_gpu_call():
    L = B.lib()
    fake = C.c_void_p(4096)
    good = B.ScoreParams(C.sizeof(B.ScoreParams), 0, 1, 1, 1, 0)
    def call(prm, rows=fake, topk=4):
        return L.slkv_score_heads_ex(C.byref(prm) if prm is not None else None, rows, 1, 1, 1, 64, 0, 4, topk, fake, None,
                                     fake, 1 << 20, None)
    assert call(None) == 1                                                        # NULL params
    assert call(B.ScoreParams(8, 0, 1, 1, 1, 0)) == 2                             # struct_size
    assert call(B.ScoreParams(C.sizeof(B.ScoreParams), 2, 1, 1, 1, 0)) == 2       # aggregation
    assert call(B.ScoreParams(C.sizeof(B.ScoreParams), 0, 1, 3, 1, 0)) == 2       # switch not 0/1
    assert call(B.ScoreParams(C.sizeof(B.ScoreParams), 0, 1, 1, 1, 7)) == 2       # reserved
    assert call(good, rows=None) == 1                                             # NULL rows
    assert call(good, topk=0) == 2                                                # topk
