"""Seeded sweep of small random problem shapes through both compression entry points: batch
size, ragged lengths (also empty, shorter than the window, within capacity), head grouping,
window, head dimension, dtype, pooling mode and kernel width, capacities from 0 to beyond the
length.  Same bar as the other parity tests."""

import numpy as np
import pytest

from paper_2508_15806_amd import binding as B
from paper_2508_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu

GROUPS = [(2, 2), (4, 2), (8, 2), (4, 1), (8, 8), (16, 4), (6, 3)]
POOLS = [(B.SLKV_POOL_MAX, 7), (B.SLKV_POOL_MAX, 3), (B.SLKV_POOL_MAX, 1), (B.SLKV_POOL_AVG, 5), (B.SLKV_POOL_NONE, 1),
         (B.SLKV_POOL_MAX, 9)]


def draw(case):
    rng = np.random.default_rng(1000 + case)
    Hq, Hkv = GROUPS[rng.integers(len(GROUPS))]
    G = Hq // Hkv
    w = int(rng.choice([4, 8, 16, 24, 32, 64]))
    while G * w > 512:
        w //= 2
    d = int(rng.choice([64, 128]))
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    pool, kern = POOLS[rng.integers(len(POOLS))]
    nb = int(rng.integers(1, 5))
    return rng, Hq, Hkv, w, d, dtype, pool, kern, nb


def lengths(rng, count, w):
    out = []
    for _ in range(count):
        r = rng.random()
        if r < 0.08:
            out.append(0)
        elif r < 0.16:
            out.append(int(rng.integers(1, w + 1)))
        else:
            out.append(int(rng.integers(w + 1, 2200)))
    return out


def capacities(rng, Hkv, w):
    return np.array([int(rng.choice([0, w, w + 1, w + int(rng.integers(2, 400)), w + int(rng.integers(2, 400)),
                                     w + int(rng.integers(400, 1500)), 5000])) for _ in range(Hkv)], dtype=np.int32)


@pytest.mark.parametrize("case", range(16))
def test_packed_batch(case):
    import parity as p
    rng, Hq, Hkv, w, d, dtype, pool, kern, nb = draw(case)
    lay = wl.make_layer((401, case), lengths(rng, nb, w), Hq, Hkv, d, w, dtype=dtype, bias_frac=0.04)
    bud = capacities(rng, Hkv, w)
    gpu = p.run_gpu(lay, bud, kern, pool)
    rep = p.compare_layer(lay, bud, gpu, kern, pool)
    print(case, Hq, Hkv, w, d, dtype, pool, kern, lay.cu_seqlens.tolist(), bud.tolist(), rep["ranked"], rep["tolerant"], flush=True)


@pytest.mark.parametrize("case", range(16, 28))
def test_ragged_cache(case):
    import parity as p
    rng, Hq, Hkv, w, d, dtype, pool, kern, nb = draw(case)
    rc = wl.make_ragged_cache((402, case), lengths(rng, nb * Hkv, w), nb, Hq, Hkv, d, w, dtype=dtype, bias_frac=0.04)
    bud = capacities(rng, Hkv, w)
    gpu = p.run_gpu_ragged(rc, bud, kern, pool)
    rep = p.compare_ragged(rc, bud, gpu, kern, pool)
    print(case, Hq, Hkv, w, d, dtype, pool, kern, np.diff(rc.in_offsets).tolist(), bud.tolist(), rep["ranked"], rep["tolerant"], flush=True)
