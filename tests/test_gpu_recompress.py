"""GPU parity of slkv_recompress_layer (Algorithm 3 on an already compacted cache) against the
float64 oracle, through the C ABI.  Same bar as for slkv_compress_layer; the carried positions
(d_pos_out) are integers and must match exactly."""

import numpy as np
import pytest

import oracle
from paper_2508_15806_amd import api
from paper_2508_15806_amd import binding as B
from paper_2508_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


def check(rc, budgets, pool_kernel=7, pool=B.SLKV_POOL_MAX, positions=True):
    import parity as p
    gpu = p.run_gpu_ragged(rc, budgets, pool_kernel, pool, positions)
    rep = p.compare_ragged(rc, budgets, gpu, pool_kernel, pool)
    print("segments %d ranked %d exact %d tolerant %d max_rel %.3g" % (
        rep["segments"], rep["ranked"], rep["exact"], rep["tolerant"], rep["max_rel"]), flush=True)
    return rep


def test_heads_of_different_lengths_bf16():
    # per-head lengths on both sides of the capacity, of the window, of the inline-gather limit
    lens = [700, 90, 16, 0, 1500, 333, 40, 2100,
            64, 65, 1000, 17, 5, 800, 801, 260]
    rc = wl.make_ragged_cache((201,), lens, 2, 16, 8, 128, 16, dtype="bf16", bias_frac=0.05)
    bud = np.array([100, 80, 16, 7, 300, 333, 64, 1025], dtype=np.int32)
    rep = check(rc, bud)
    assert rep["ranked"] >= 6


@pytest.mark.parametrize("Hq,Hkv,w,d,dtype", [(4, 2, 8, 64, "f32"), (8, 2, 32, 128, "bf16"), (8, 8, 24, 64, "bf16"),
                                              (8, 2, 32, 128, "f16"), (8, 2, 32, 128, "bf16_kv8")])
def test_shapes(Hq, Hkv, w, d, dtype):
    rng = np.random.default_rng(7)
    lens = rng.integers(w + 1, 900, size=3 * Hkv).tolist()
    rc = wl.make_ragged_cache((202, Hq, w), lens, 3, Hq, Hkv, d, w, dtype=dtype, bias_frac=0.04)
    bud = np.array([w + 20 + 37 * h for h in range(Hkv)], dtype=np.int32)
    check(rc, bud, positions=(dtype != "f32"))


def test_offsets_need_not_start_at_zero():
    rc = wl.make_ragged_cache((203,), [50, 400, 300, 120], 2, 4, 2, 128, 16, dtype="bf16", bias_frac=0.05)
    # view of the cache that skips the first segment: one sequence is left (segments 2 and 3)
    import parity as p
    sub = wl.RaggedCache(rc.dtype, 1, rc.Hq, rc.Hkv, rc.d, rc.w, rc.in_offsets[2:], rc.qwin[1:], rc.k_rows, rc.v_rows,
                         rc.pos_in)
    bud = np.array([100, 60], dtype=np.int32)
    gpu = p.run_gpu_ragged(sub, bud)
    ref = oracle.recompress_layer(sub.qwin, sub.k_rows, sub.v_rows, sub.in_offsets, bud, sub.w, pos_in=sub.pos_in)
    assert np.array_equal(gpu["kept"], np.concatenate([s["kept_idx"] for s in ref["segments"]]))
    assert np.array_equal(gpu["k_out"], ref["k_out"]) and np.array_equal(gpu["pos_out"], ref["pos_out"])


def test_prefill_decode_chain_matches_the_oracle_chain():
    # prefill compression, 48 generated tokens appended to every head, re-compression: positions
    # carried through both steps equal those of the oracle's chain
    import torch
    import parity as p
    w, Hq, Hkv, d = 16, 8, 4, 128
    lay = wl.make_layer((204,), [1200, 500], Hq, Hkv, d, w, dtype="bf16", bias_frac=0.05)
    bud = np.array([200, 64, 333, 90], dtype=np.int32)
    first = p.run_gpu(lay, bud)
    ref1 = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, bud, w)
    assert np.array_equal(first["kept"], np.concatenate([s["kept_idx"] for s in ref1["segments"]]))
    # grow every segment by `new` rows (host side bookkeeping, same for both chains)
    new = 48
    extra = wl.make_ragged_cache((205,), [new] * (2 * Hkv), 2, Hq, Hkv, d, w, dtype="bf16")
    rows_k, rows_v, pos, offs = [], [], [], [0]
    for s in range(2 * Hkv):
        b = s // Hkv
        o0, o1 = int(ref1["out_offsets"][s]), int(ref1["out_offsets"][s + 1])
        n_b = int(lay.cu_seqlens[b + 1] - lay.cu_seqlens[b])
        rows_k += [first["k_out"][o0:o1], extra.k_rows[s * new:(s + 1) * new]]
        rows_v += [first["v_out"][o0:o1], extra.v_rows[s * new:(s + 1) * new]]
        pos += [first["kept"][o0:o1], np.arange(n_b, n_b + new, dtype=np.int32)]
        offs.append(offs[-1] + o1 - o0 + new)
    rc = wl.RaggedCache("bf16", 2, Hq, Hkv, d, w, np.asarray(offs, dtype=np.int64), extra.qwin,
                        np.concatenate(rows_k), np.concatenate(rows_v), np.concatenate(pos).astype(np.int32))
    rep = check(rc, bud)
    assert rep["ranked"] >= 6


def test_config6_shape_sample():
    # the benchmark's decode-time workload at a small batch
    inf = wl.config3_inf()
    row = wl.config5_layer_row(inf)
    bud = B.slkv_allocate_budgets(inf, 8, 256, 16)[row]
    lens = [oracle.kept_count(32768, 64, int(c)) + 128 for c in bud]
    rc = wl.config6(lens, batch=3)
    rep = check(rc, bud)
    assert rep["segments"] == 24


def test_hundreds_of_segments_use_the_device_resident_table():
    rng = np.random.default_rng(11)
    Hkv, Bn, w = 4, 75, 16                                     # 300 segments
    lens = rng.integers(0, 700, size=Bn * Hkv)
    lens[::17] = 0
    lens[5::23] = w
    rc = wl.make_ragged_cache((206,), lens.tolist(), Bn, 8, Hkv, 64, w, dtype="bf16", bias_frac=0.04)
    bud = np.array([60, 300, 16, 128], dtype=np.int32)
    rep = check(rc, bud)
    assert rep["segments"] == 300 and rep["ranked"] > 100


def test_cache_without_rows():
    # every segment empty: NULL input buffers (torch's empty tensors) are accepted, offsets are written
    import torch
    call = api.RaggedCall("bf16", 2, 4, 2, 128, 16, np.zeros(5, dtype=np.int64), np.array([40, 7], dtype=np.int32))
    assert call.total_kept == 0
    q = torch.zeros((2, 4, 16, 128), dtype=torch.bfloat16, device="cuda")
    empty = torch.empty((0, 128), dtype=torch.bfloat16, device="cuda")
    call.out_offsets.fill_(-1)
    call.run(q, empty, empty, torch.empty((0,), dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert (call.out_offsets.cpu().numpy() == 0).all()
