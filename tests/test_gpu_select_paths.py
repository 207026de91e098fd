"""Both selection kernels (one workgroup per segment; histories cut into blocks with a per-segment
ticket) on the same shapes: SLKV_SELECT in the environment forces one of them, the library reads
it at every call.  Same bar as the other parity tests; the two must also agree bit for bit."""

import os

import numpy as np
import pytest

from paper_2508_15806_amd import binding as B
from paper_2508_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["resident", "blocks"])
def select_path(request):
    old = os.environ.get("SLKV_SELECT")
    os.environ["SLKV_SELECT"] = request.param
    yield request.param
    if old is None:
        del os.environ["SLKV_SELECT"]
    else:
        os.environ["SLKV_SELECT"] = old


def run(lay, bud, kernel=7, pool=B.SLKV_POOL_MAX):
    import parity as p
    gpu = p.run_gpu(lay, bud, kernel, pool)
    rep = p.compare_layer(lay, bud, gpu, kernel, pool)
    return gpu, rep


def test_config2(select_path):
    lay = wl.config2()
    bud = B.slkv_allocate_budgets(lay.meta["inf"], lay.Hkv, lay.meta["avg"], lay.meta["fixed"])[0]
    gpu, rep = run(lay, bud)
    assert rep["ranked"] == 8 and rep["tolerant"] == 0


@pytest.mark.parametrize("pool,kernel", [(B.SLKV_POOL_MAX, 7), (B.SLKV_POOL_MAX, 13), (B.SLKV_POOL_AVG, 5), (B.SLKV_POOL_NONE, 1)])
def test_several_blocks_per_segment_and_ragged_tails(select_path, pool, kernel):
    # histories of 2.4 and 5.1 blocks of 4096 positions next to short and unranked segments
    lay = wl.make_layer((601, kernel), [9900 + 16, 300, 21000 + 16 + 5, 10], 4, 2, 64, 16, dtype="bf16", bias_frac=0.03)
    gpu, rep = run(lay, np.array([700, 3000], dtype=np.int32), kernel, pool)
    assert rep["ranked"] == 4 and rep["tolerant"] == 0


@pytest.mark.parametrize("n,protos,budget", [(9016, 2, 2000), (9016, 2, 6000), (30016, 3, 14000), (3016, 1, 3015)])
def test_tie_groups(select_path, n, protos, budget):
    w = 16
    lay = wl.make_layer((602, n, protos), [n], 2, 1, 64, w, dtype="bf16")
    m = n - w
    lay.k[:, :m, :] = lay.k[:, :protos, :][:, np.arange(m) % protos, :]
    gpu, rep = run(lay, np.array([budget], dtype=np.int32), 1, B.SLKV_POOL_NONE)
    assert rep["ranked"] == 1 and rep["tolerant"] == 0


def test_paths_agree_bit_for_bit():
    import parity as p
    lay = wl.make_layer((603,), [12000, 5000, 77], 8, 4, 128, 32, dtype="bf16", bias_frac=0.03)
    bud = np.array([100, 1500, 32, 6000], dtype=np.int32)
    outs = {}
    old = os.environ.get("SLKV_SELECT")
    try:
        for mode in ("resident", "blocks"):
            os.environ["SLKV_SELECT"] = mode
            outs[mode] = p.run_gpu(lay, bud)
    finally:
        if old is None:
            os.environ.pop("SLKV_SELECT", None)
        else:
            os.environ["SLKV_SELECT"] = old
    for key in ("offsets", "kept", "k_out", "v_out", "pooled"):
        assert np.array_equal(outs["resident"][key], outs["blocks"][key]), key


def test_one_long_history_among_many_short_ones(select_path):
    # block-wise compaction with one grid row over all blocks (a grid row per segment would be mostly
    # empty here), segments that are not ranked in between, more than 64 segments (device table)
    lens = [45000] + [150 + 37 * (i % 9) for i in range(70)] + [20]
    lay = wl.make_layer((604,), lens, 2, 1, 64, 16, dtype="bf16", bias_frac=0.03)
    gpu, rep = run(lay, np.array([180], dtype=np.int32))
    assert rep["segments"] == len(lens) and rep["ranked"] >= 40 and rep["tolerant"] == 0
