"""slkv_compress_layer allocates nothing, copies nothing and never synchronises, so a call can be
recorded into a HIP graph.  Every replay must reproduce the eager result for the inputs that are
in the buffers at replay time."""

import numpy as np
import pytest

from paper_2508_15806_amd import api
from paper_2508_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


def outputs(call):
    return [api.to_host(call.k_out).copy(), api.to_host(call.v_out).copy(), call.kept_idx.cpu().numpy().copy(),
            call.out_offsets.cpu().numpy().copy()]


def test_captured_call_replays_like_eager():
    import torch
    Hq, Hkv, d, w = 8, 2, 128, 16
    lays = [wl.make_layer((301, i), [2500, 700], Hq, Hkv, d, w, dtype="bf16", bias_frac=0.05) for i in range(3)]
    bud = np.array([300, 77], dtype=np.int32)
    call = api.LayerCall("bf16", 2, Hq, Hkv, d, w, lays[0].cu_seqlens, bud)
    q = api.to_device(lays[0].qwin, "bf16")
    k = api.to_device(lays[0].k, "bf16")
    v = api.to_device(lays[0].v, "bf16")
    # eager references for the three input sets
    refs = []
    for lay in lays:
        q.copy_(api.to_device(lay.qwin, "bf16")); k.copy_(api.to_device(lay.k, "bf16")); v.copy_(api.to_device(lay.v, "bf16"))
        call.run(q, k, v)
        torch.cuda.synchronize()
        refs.append(outputs(call))
    assert not np.array_equal(refs[0][2], refs[1][2])
    # capture one call on a side stream
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        call.run(q, k, v)                       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        call.run(q, k, v)
    # replays with eager work and synchronisations in between
    for rep in range(2):
        for i, lay in enumerate(lays):
            q.copy_(api.to_device(lay.qwin, "bf16")); k.copy_(api.to_device(lay.k, "bf16")); v.copy_(api.to_device(lay.v, "bf16"))
            call.kept_idx.fill_(-1)
            call.k_out.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = outputs(call)
            for a, b in zip(got, refs[i]):
                assert np.array_equal(a, b), (rep, i)
