"""GPU parity of slkv_compress_layer against the float64 oracle, through the C ABI.

Bar: out offsets and kept-index sets bit-exact (positions whose pooled score is within the
tolerance of the k-th score may differ and are reported); gathered K/V bit-exact; importance
and pooled scores within 2e-3 (bf16 inputs) / 1e-5 (fp32 inputs) relative."""

import numpy as np
import pytest

import oracle
from paper_2508_15806_amd import binding as B
from paper_2508_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


def parity():
    import parity as p
    return p


def budgets_for(lay, inf=None, avg=None, fixed=None):
    inf = lay.meta["inf"] if inf is None else inf
    avg = lay.meta["avg"] if avg is None else avg
    fixed = lay.meta["fixed"] if fixed is None else fixed
    got = B.slkv_allocate_budgets(inf, lay.Hkv, avg, fixed)
    assert got.tolist() == oracle.allocate_budgets(np.asarray(inf).tolist(), lay.Hq, lay.Hkv, avg, fixed)
    return got


def check(lay, budgets, pool_kernel=7, pool=B.SLKV_POOL_MAX, require_exact=False, token_major=False):
    p = parity()
    gpu = p.run_gpu(lay, budgets, pool_kernel, pool, token_major=token_major)
    rep = p.compare_layer(lay, budgets, gpu, pool_kernel, pool)
    print("segments %d ranked %d exact %d tolerant %d max_rel %.3g diffs %s" % (
        rep["segments"], rep["ranked"], rep["exact"], rep["tolerant"], rep["max_rel"], rep["diffs"][:4]), flush=True)
    if require_exact:
        assert rep["tolerant"] == 0
    return rep


def test_config1_fp32():
    lay = wl.config1()
    rep = check(lay, budgets_for(lay)[0], require_exact=True)
    assert rep["ranked"] == 4


def test_config2_bf16():
    lay = wl.config2()
    bud = budgets_for(lay)[0]
    assert int(bud.sum()) == 128 * 8
    rep = check(lay, bud, require_exact=True)
    assert rep["ranked"] == 8


@pytest.mark.parametrize("Hq,Hkv,w,d", [(2, 2, 16, 128), (4, 2, 16, 128), (8, 2, 16, 128), (8, 2, 32, 128),
                                        (16, 2, 32, 128), (4, 4, 24, 64), (8, 2, 20, 64), (32, 8, 16, 64),
                                        (16, 2, 64, 128), (16, 2, 64, 64), (8, 1, 48, 128), (8, 2, 64, 64)])
def test_bf16_row_shapes_and_ragged_tails(Hq, Hkv, w, d):
    # lengths chosen so that the history is not a multiple of the 32-key MFMA tile
    lay = wl.make_layer((101, Hq, w, d), [1000 + w + 7, 333 + w], Hq, Hkv, d, w, dtype="bf16", bias_frac=0.03)
    bud = np.array([w + 40 + 13 * h for h in range(Hkv)], dtype=np.int32)
    check(lay, bud)


@pytest.mark.parametrize("Hq,Hkv,w,d", [(2, 2, 16, 128), (8, 2, 32, 128), (4, 4, 24, 64), (32, 8, 16, 64),
                                        (16, 4, 64, 128), (16, 2, 64, 64)])
def test_fp16_row_shapes_and_ragged_tails(Hq, Hkv, w, d):
    # IEEE half inputs through the same MFMA kernels (32 to 512 rows per KV head, both head dims)
    lay = wl.make_layer((131, Hq, w, d), [1000 + w + 7, 333 + w], Hq, Hkv, d, w, dtype="f16", bias_frac=0.03)
    assert lay.k.dtype == np.float16
    bud = np.array([w + 40 + 13 * h for h in range(Hkv)], dtype=np.int32)
    check(lay, bud)


def test_fp16_long_history_and_token_major():
    lay = wl.make_layer((132,), [40000 + 64 + 9, 700], 8, 2, 128, 64, dtype="f16", bias_frac=0.02)
    rep = check(lay, np.array([900, 150], dtype=np.int32))                  # the 700-token sequence fits the first head's capacity
    assert rep["ranked"] == 3 and rep["tolerant"] == 0
    lay = wl.make_layer((133,), [1500 + 11, 0, 260], 8, 4, 128, 16, dtype="f16", bias_frac=0.04)
    rep = check(lay, np.array([300, 16, 90, 2000], dtype=np.int32), token_major=True)
    assert rep["ranked"] == 3 and rep["tolerant"] == 0


@pytest.mark.parametrize("Hq,Hkv,w,d", [(2, 2, 16, 128), (8, 2, 32, 128), (4, 4, 24, 64), (16, 4, 64, 128), (16, 2, 64, 64)])
def test_e4m3_keys_and_values_row_shapes(Hq, Hkv, w, d):
    # bf16 queries against keys / values stored as E4M3 bytes (widened to bf16 inside the kernels, exactly)
    lay = wl.make_layer((141, Hq, w, d), [1000 + w + 7, 333 + w], Hq, Hkv, d, w, dtype="bf16_kv8", bias_frac=0.03)
    assert lay.k.dtype == np.uint8 and lay.qwin.dtype == np.uint16
    bud = np.array([w + 40 + 13 * h for h in range(Hkv)], dtype=np.int32)
    check(lay, bud)


def test_e4m3_every_code_long_history_and_token_major():
    lay = wl.make_layer((142,), [40000 + 64 + 9, 700], 8, 2, 128, 64, dtype="bf16_kv8", bias_frac=0.02)
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)      # every finite code, subnormals included
    lay.k[0, :codes.size * 4, :] = np.resize(codes, (codes.size * 4, 128))
    rep = check(lay, np.array([900, 150], dtype=np.int32))
    assert rep["ranked"] == 3 and rep["tolerant"] == 0
    lay = wl.make_layer((143,), [1500 + 11, 0, 260], 8, 4, 128, 16, dtype="bf16_kv8", bias_frac=0.04)
    rep = check(lay, np.array([300, 16, 90, 2000], dtype=np.int32), token_major=True)
    assert rep["ranked"] == 3 and rep["tolerant"] == 0


@pytest.mark.parametrize("Hq,Hkv,w,d", [(2, 2, 8, 64), (4, 2, 32, 128), (8, 1, 40, 64)])
def test_fp32_shapes(Hq, Hkv, w, d):
    lay = wl.make_layer((102, Hq, w, d), [700 + w + 5, 90], Hq, Hkv, d, w, dtype="f32", bias_frac=0.03)
    bud = np.array([w + 30 + 11 * h for h in range(Hkv)], dtype=np.int32)
    check(lay, bud)


def test_edge_segments():
    # empty sequence, n <= w, n <= capacity, capacity <= window, capacity == n - 1
    w = 16
    lay = wl.make_layer((103,), [0, 10, 16, 200, 17, 300], 4, 2, 128, w, dtype="bf16", bias_frac=0.05)
    for bud in ([200, 5], [299, 16], [17, 0], [1000, 1000]):
        check(lay, np.array(bud, dtype=np.int32))


@pytest.mark.parametrize("pool,kernel", [(B.SLKV_POOL_MAX, 1), (B.SLKV_POOL_MAX, 3), (B.SLKV_POOL_MAX, 13),
                                         (B.SLKV_POOL_AVG, 7), (B.SLKV_POOL_NONE, 7)])
def test_pool_modes(pool, kernel):
    lay = wl.make_layer((104, kernel), [900], 8, 2, 128, 16, dtype="bf16", bias_frac=0.05)
    check(lay, np.array([100, 333], dtype=np.int32), kernel, pool)


def test_heavy_ties_are_cut_by_lowest_position():
    # identical keys everywhere: every importance score ties, so the kept set must be the lowest positions
    lay = wl.make_layer((105,), [600], 4, 2, 128, 16, dtype="bf16")
    lay.k[:, :, :] = lay.k[:, :1, :]
    rep = check(lay, np.array([100, 50], dtype=np.int32), require_exact=True)
    assert rep["ranked"] == 2
    # two alternating key values: long plateaus after max pooling
    lay = wl.make_layer((106,), [1500], 4, 2, 128, 16, dtype="bf16")
    lay.k[:, 1::2, :] = lay.k[:, 1:2, :]
    lay.k[:, 0::2, :] = lay.k[:, 0:1, :]
    check(lay, np.array([200, 700], dtype=np.int32), require_exact=True)


@pytest.mark.parametrize("n,protos,budget", [(5016, 5, 1500), (9016, 2, 2000), (9016, 2, 6000), (70008, 2, 40000),
                                             (3016, 1, 3015)])
def test_tie_groups_of_every_size(n, protos, budget):
    # History keys drawn from a few prototypes, no pooling: the scores form `protos` groups of equal
    # values, so the threshold falls inside a tie group of hundreds to tens of thousands of entries
    # (in-LDS candidate list, list overflow, several compaction rounds).
    w = 16
    lay = wl.make_layer((109, n, protos), [n], 2, 1, 64, w, dtype="bf16")
    m = n - w
    lay.k[:, :m, :] = lay.k[:, :protos, :][:, np.arange(m) % protos, :]
    rep = check(lay, np.array([budget], dtype=np.int32), 1, B.SLKV_POOL_NONE, require_exact=True)
    assert rep["ranked"] == 1


def test_inline_and_separate_gather_in_one_launch():
    # kept-row counts on both sides of the limit up to which the selection kernel copies rows itself
    lay = wl.make_layer((110,), [3000, 1500, 40], 8, 4, 128, 16, dtype="bf16", bias_frac=0.05)
    check(lay, np.array([256, 257, 16, 2900], dtype=np.int32))
    lay = wl.make_layer((111,), [2100], 4, 2, 64, 8, dtype="f32", bias_frac=0.05)
    check(lay, np.array([256, 1500], dtype=np.int32))


def test_many_segments_span_several_launch_groups():
    lens = [150 + 7 * i for i in range(40)]                        # 40 sequences x 2 heads = 80 segments
    lay = wl.make_layer((107,), lens, 4, 2, 64, 8, dtype="bf16", bias_frac=0.05)
    check(lay, np.array([40, 100], dtype=np.int32))


def test_two_runs_are_bit_identical():
    p = parity()
    lay = wl.config2()
    bud = budgets_for(lay)[0]
    a = p.run_gpu(lay, bud)
    b = p.run_gpu(lay, bud)
    for key in ("offsets", "kept", "k_out", "v_out", "importance", "pooled"):
        assert np.array_equal(a[key], b[key]), key


def test_long_segment_multi_round_compaction():
    # history longer than one compaction round (128 * 1024 positions) and than 2^16 kept rows
    lay = wl.make_layer((108,), [140000], 2, 1, 64, 8, dtype="bf16", bias_frac=0.01)
    check(lay, np.array([70008], dtype=np.int32))


# layers 0, 1, 5 hold no spike head of the INF_sc map; 7, 10 and 30 do (capacities of 320-440 at
# average 64 and of 7800-9000 at average 1024, next to heads at the fixed part)
@pytest.mark.parametrize("layer", [0, 1, 5, 7, 10, 30])
def test_config3_layers_all_budgets(layer):
    p = parity()
    lay = wl.config3_layer(layer)
    inf = wl.config3_inf()
    cache = {}                                   # oracle scores do not depend on the budgets
    for avg in wl.C3_BUDGETS:
        bud = budgets_for(lay, inf, avg, 16)[layer]
        gpu = p.run_gpu(lay, bud)
        ref = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, bud, lay.w, 7, score_cache=cache)
        rep = p.compare_layer(lay, bud, gpu, ref=ref)
        print("c3 layer %d avg %d: ranked %d exact %d tolerant %d max_rel %.3g" % (
            layer, avg, rep["ranked"], rep["exact"], rep["tolerant"], rep["max_rel"]), flush=True)
        assert rep["tolerant"] == 0 and rep["exact"] == rep["segments"] == 8
        assert rep["ranked"] == sum(1 for c in bud if c > lay.w)
        if layer in (7, 10, 30):
            assert rep["ranked"] > 0, "a spike-bearing layer ranks at least its spike head at every budget"
        if avg == 1024:
            assert rep["ranked"] == 8


def test_config5_ragged_long_context():
    p = parity()
    lay = wl.config5()
    inf = wl.config3_inf()
    row = wl.config5_layer_row(inf)
    bud = budgets_for(lay, inf, 512, 64)[row]
    gpu = p.run_gpu(lay, bud)
    rep = p.compare_layer(lay, bud, gpu)
    print("c5: segments %d ranked %d exact %d tolerant %d max_rel %.3g" % (
        rep["segments"], rep["ranked"], rep["exact"], rep["tolerant"], rep["max_rel"]), flush=True)
    assert rep["segments"] == 32 and rep["tolerant"] == 0 and rep["exact"] == 32


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_token_major_keys_and_padded_value_rows(dtype):
    # K as [T][Hkv][d] (token stride Hkv*d, head stride d), V with rows padded to d + 24 elements:
    # the strides of the two tensors differ and neither is the head-major default
    lay = wl.make_layer((113, dtype == "bf16"), [1500 + 11, 0, 260], 8, 4, 128 if dtype == "bf16" else 64, 16,
                        dtype=dtype, bias_frac=0.04)
    bud = np.array([300, 16, 90, 2000], dtype=np.int32)
    rep = check(lay, bud, token_major=True)
    assert rep["ranked"] == 3 and rep["tolerant"] == 0


def test_extreme_logits_take_the_running_maximum_path():
    # The first 64 history keys of every head are zero and the later ones are large and aligned with
    # the queries: their logits exceed the first ones by far more than fp32 exponent range allows
    # for a sum referenced to the first logits, so the statistics pass has to repeat its chunk
    # with the running maximum.  The softmax then concentrates on the late keys.
    w, Hq, Hkv, d = 16, 4, 2, 128
    lay = wl.make_layer((112,), [1200, 300], Hq, Hkv, d, w, dtype="bf16")
    three = wl.to_bf16_bits(np.full((d,), 3.0, dtype=np.float32))
    small = wl.to_bf16_bits(np.random.default_rng(1).standard_normal((Hkv, 1500, d)).astype(np.float32) * 0.01)
    lay.qwin[:] = three
    lay.k[:] = small
    lay.k[:, 500:560, :] = three            # logits 9 * 128 / sqrt(128) = 101.8 nats = 146.9 in base 2
    lay.k[:, 1200:1264, :] = 0              # second sequence: zero keys first, then large ones
    lay.k[:, 1300:1360, :] = three
    # capacities below the number of large keys: everything else underflows in fp32 on the GPU
    # (its true weight is about e^-100), so only the large keys can be ranked
    rep = check(lay, np.array([w + 50, w + 8], dtype=np.int32))
    assert rep["ranked"] == 4


def test_extreme_logits_with_256_rows_per_head():
    # the same situation on the shape of the long-context configurations (4 query heads x 64 window rows per KV head:
    # the statistics pass that overlaps its exponentials with the next sub-tile's MFMAs), chunk tails included
    w, Hq, Hkv, d = 64, 8, 2, 128
    lay = wl.make_layer((114,), [2100 + 37, 700], Hq, Hkv, d, w, dtype="bf16")
    three = wl.to_bf16_bits(np.full((d,), 3.0, dtype=np.float32))
    small = wl.to_bf16_bits(np.random.default_rng(2).standard_normal((Hkv, 2837, d)).astype(np.float32) * 0.01)
    lay.qwin[:] = three
    lay.k[:] = small
    lay.k[:, 900:980, :] = three
    lay.k[:, 2137 + 300:2137 + 380, :] = three
    rep = check(lay, np.array([w + 60, w + 9], dtype=np.int32))
    assert rep["ranked"] == 4


def test_batch_without_tokens():
    # every sequence empty: the inputs and outputs have no rows (torch hands out NULL pointers for
    # them); the call still has to succeed and write the offsets
    import torch
    from paper_2508_15806_amd import api
    call = api.LayerCall("bf16", 3, 4, 2, 128, 16, np.zeros(4, dtype=np.int64), np.array([40, 7], dtype=np.int32))
    assert call.total_kept == 0
    q = torch.zeros((3, 4, 16, 128), dtype=torch.bfloat16, device="cuda")
    empty = torch.empty((2, 0, 128), dtype=torch.bfloat16, device="cuda")
    call.out_offsets.fill_(-1)
    B.slkv_compress_layer(call.layer, q, empty, empty, empty.reshape(0, 128), empty.reshape(0, 128),
                          torch.empty((0,), dtype=torch.int32, device="cuda"), call.workspace, call.out_offsets)
    torch.cuda.synchronize()
    assert (call.out_offsets.cpu().numpy() == 0).all()
