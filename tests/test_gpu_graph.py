"""slkv_compress_layer allocates nothing, copies nothing and never synchronises, so a call can be
recorded into a HIP graph.  Every replay must reproduce the eager result for the inputs that are
in the buffers at replay time."""

import numpy as np
import pytest

from paper_2508_15806_amd import api
from paper_2508_15806_amd import binding as B
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
    # capture one call on a side stream (the device's one-time set-up is not a stream operation)
    B.slkv_init()
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


def test_captured_ragged_call_with_device_table_replays_like_eager():
    # more than 64 segments: the call also launches the small kernels that write the segment table
    import torch
    rng = np.random.default_rng(3)
    Hkv, Bn, w, d, Hq = 4, 24, 16, 64, 8                         # 96 segments
    lens = rng.integers(w + 1, 500, size=Bn * Hkv).tolist()
    rcs = [wl.make_ragged_cache((302, i), lens, Bn, Hq, Hkv, d, w, dtype="bf16", bias_frac=0.04) for i in range(2)]
    bud = np.array([60, 200, 16, 100], dtype=np.int32)
    call = api.RaggedCall("bf16", Bn, Hq, Hkv, d, w, rcs[0].in_offsets, bud)
    q = api.to_device(rcs[0].qwin, "bf16")
    k = api.to_device(rcs[0].k_rows, "bf16")
    v = api.to_device(rcs[0].v_rows, "bf16")
    pos = torch.from_numpy(rcs[0].pos_in).cuda()

    def load(rc):
        q.copy_(api.to_device(rc.qwin, "bf16")); k.copy_(api.to_device(rc.k_rows, "bf16")); v.copy_(api.to_device(rc.v_rows, "bf16"))
        pos.copy_(torch.from_numpy(rc.pos_in).cuda())

    def outs():
        return [api.to_host(call.k_out).copy(), call.kept_idx.cpu().numpy().copy(), call.pos_out.cpu().numpy().copy()]
    refs = []
    for rc in rcs:
        load(rc)
        call.run(q, k, v, pos)
        torch.cuda.synchronize()
        refs.append(outs())
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        call.run(q, k, v, pos)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        call.run(q, k, v, pos)
    for rep in range(2):
        for i, rc in enumerate(rcs):
            load(rc)
            call.kept_idx.fill_(-1)
            call.workspace.zero_()                               # the table in the workspace is rewritten by the replay
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for a, b in zip(outs(), refs[i]):
                assert np.array_equal(a, b), (rep, i)


def test_calls_on_two_streams_do_not_interfere():
    # Calls whose buffers are disjoint may overlap on the GPU (streams of the default priority): each
    # keeps its own workspace, and the library holds no device state that two calls share.
    import torch
    Hq, Hkv, d, w = 16, 4, 128, 32
    lays = [wl.make_layer((303, i), [6000, 2500], Hq, Hkv, d, w, dtype="bf16", bias_frac=0.05) for i in range(4)]
    buds = [np.array([300, 77, 1000, 40], dtype=np.int32), np.array([64, 500, 33, 200], dtype=np.int32)]
    calls = [api.LayerCall("bf16", 2, Hq, Hkv, d, w, lay.cu_seqlens, buds[i & 1]) for i, lay in enumerate(lays)]
    dev = [(api.to_device(lay.qwin, "bf16"), api.to_device(lay.k, "bf16"), api.to_device(lay.v, "bf16")) for lay in lays]
    refs = []
    for call, (q, k, v) in zip(calls, dev):
        call.run(q, k, v)
        torch.cuda.synchronize()
        refs.append(outputs(call))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(4):
        for call in calls:
            call.kept_idx.fill_(-1)
            call.k_out.zero_()
        torch.cuda.synchronize()
        for i, (call, (q, k, v)) in enumerate(zip(calls, dev)):
            with torch.cuda.stream(streams[i & 1]):
                call.run(q, k, v)
        torch.cuda.synchronize()
        for i, call in enumerate(calls):
            for a, b in zip(outputs(call), refs[i]):
                assert np.array_equal(a, b), (rep, i)


def test_captured_block_wise_selection_replays_like_eager():
    # the selection of long histories is six launches that hand their state on through the workspace
    # (digit, list length, threshold, per-block counts): every replay has to start it afresh
    import os
    import torch
    Hq, Hkv, d, w = 4, 2, 64, 16
    lays = [wl.make_layer((304, i), [9000, 2600], Hq, Hkv, d, w, dtype="bf16", bias_frac=0.05) for i in range(3)]
    bud = np.array([500, 90], dtype=np.int32)
    old = os.environ.get("SLKV_SELECT")
    os.environ["SLKV_SELECT"] = "blocks"
    try:
        call = api.LayerCall("bf16", 2, Hq, Hkv, d, w, lays[0].cu_seqlens, bud)
        q = api.to_device(lays[0].qwin, "bf16")
        k = api.to_device(lays[0].k, "bf16")
        v = api.to_device(lays[0].v, "bf16")
        refs = []
        for lay in lays:
            q.copy_(api.to_device(lay.qwin, "bf16")); k.copy_(api.to_device(lay.k, "bf16")); v.copy_(api.to_device(lay.v, "bf16"))
            call.run(q, k, v)
            torch.cuda.synchronize()
            refs.append(outputs(call))
        assert not np.array_equal(refs[0][2], refs[1][2])
        B.slkv_init()
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            call.run(q, k, v)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            call.run(q, k, v)
    finally:
        if old is None:
            os.environ.pop("SLKV_SELECT", None)
        else:
            os.environ["SLKV_SELECT"] = old
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
