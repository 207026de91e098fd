"""slkv_compress_layer_static (the entry point that allocates nothing: its scratch is a buffer inside
the library) against slkv_compress_layer with a caller-owned workspace, through the C ABI.
Two calls in a row on the same GPU, the second with a smaller input: every output must be
bit-identical (the shared scratch keeps the first call's contents, nothing stale may leak)."""

import numpy as np
import pytest

from paper_2508_15806_amd import api
from paper_2508_15806_amd import binding as B
from paper_2508_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_both(lay, bud, pool_kernel=7, pool=B.SLKV_POOL_MAX):
    import torch
    ref = api.LayerCall(lay.dtype, lay.B, lay.Hq, lay.Hkv, lay.d, lay.w, lay.cu_seqlens, bud, pool_kernel, pool,
                        debug_scores=True)
    q, k, v = (api.to_device(x, lay.dtype) for x in (lay.qwin, lay.k, lay.v))
    ref.run(q, k, v)
    torch.cuda.synchronize()
    want = [api.to_host(ref.k_out).copy(), api.to_host(ref.v_out).copy(), ref.kept_idx.cpu().numpy().copy(),
            ref.out_offsets.cpu().numpy().copy(), ref.importance.cpu().numpy().copy(), ref.pooled.cpu().numpy().copy()]
    got = api.LayerCall(lay.dtype, lay.B, lay.Hq, lay.Hkv, lay.d, lay.w, lay.cu_seqlens, bud, pool_kernel, pool,
                        debug_scores=True)
    got.workspace = None                                    # never handed to the library
    got.kept_idx.fill_(-7)
    got.k_out.zero_()
    got.v_out.zero_()
    B.slkv_compress_layer_static(got.layer, q, k, v, got.k_out, got.v_out, got.kept_idx, got.out_offsets,
                                 got.importance, got.pooled)
    torch.cuda.synchronize()
    have = [api.to_host(got.k_out), api.to_host(got.v_out), got.kept_idx.cpu().numpy(), got.out_offsets.cpu().numpy(),
            got.importance.cpu().numpy(), got.pooled.cpu().numpy()]
    names = ["k_out", "v_out", "kept_idx", "out_offsets", "importance", "pooled"]
    for name, a, b in zip(names, have, want):
        assert np.array_equal(a, b), name
    return int(ref.total_kept)


def test_static_scratch_matches_workspace_entry_point_twice():
    # first call: several key chunks per segment, ragged tails, inline and separate gather
    lay = wl.make_layer((501,), [5000 + 37, 1200], 8, 2, 128, 32, dtype="bf16", bias_frac=0.03)
    kept1 = run_both(lay, np.array([700, 150], dtype=np.int32))
    # second call, smaller input (fewer chunks, fewer rows): nothing of the first may show
    lay2 = wl.make_layer((502,), [900, 40], 4, 2, 64, 16, dtype="bf16", bias_frac=0.05)
    kept2 = run_both(lay2, np.array([100, 60], dtype=np.int32), 3, B.SLKV_POOL_AVG)
    assert kept2 < kept1
    # and an fp32 call after the bf16 ones
    lay3 = wl.make_layer((503,), [700], 4, 4, 64, 8, dtype="f32", bias_frac=0.05)
    run_both(lay3, np.array([64, 20, 300, 9], dtype=np.int32))


def test_static_scratch_rejects_calls_beyond_its_size():
    import torch
    # 8 KV heads x 400000 tokens: importance + pooled alone need 25 MB
    n = 400000
    layer = B.Layer(B.SLKV_BF16, 1, 8, 8, 128, 16, [0, n], [100] * 8, (128, n * 128), (128, n * 128))
    assert B.slkv_workspace_bytes(layer) > (8 << 20)
    dummy = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.SlkvError) as ei:
        B.slkv_compress_layer_static(layer, dummy, dummy, dummy, dummy.view(32, 128), dummy.view(32, 128), dummy)
    assert ei.value.status == 5
