"""Shared comparison logic for the GPU parity tests (imports the oracle; test-only)."""

import numpy as np

import oracle
from paper_2508_15806_amd import api
from paper_2508_15806_amd import binding as B

TOL = {"bf16": 2e-3, "f16": 2e-3, "bf16_kv8": 2e-3, "f32": 1e-5}      # relative tolerance on importance scores (task statement; the other 16-bit and 8-bit inputs as bf16)

BAND = 4096                            # guard bytes on either side of every output / workspace buffer
SENTINEL = 0xA5


class Guarded:
    """Re-homes the output and workspace tensors of a LayerCall / RaggedCall inside larger
    sentinel-filled allocations, so that a kernel writing outside a buffer is caught even when
    the stray write would land in a neighbouring allocation.  check() runs on the host."""

    NAMES = ("k_out", "v_out", "kept_idx", "pos_out", "out_offsets", "workspace", "importance", "pooled")

    def __init__(self, call):
        import torch
        self.full = {}
        for name in self.NAMES:
            t = getattr(call, name, None)
            if t is None:
                continue
            nbytes = t.numel() * t.element_size()
            full = torch.full((BAND + nbytes + BAND,), SENTINEL, dtype=torch.uint8, device=t.device)
            inner = full[BAND:BAND + nbytes].view(t.dtype).view(t.shape)
            if name in ("workspace", "importance", "pooled"):
                inner.zero_()
            setattr(call, name, inner)
            self.full[name] = (full, nbytes)

    def check(self):
        for name, (full, nbytes) in self.full.items():
            host = full.cpu().numpy()
            assert (host[:BAND] == SENTINEL).all(), "write below the start of %s" % name
            assert (host[BAND + nbytes:] == SENTINEL).all(), "write past the end of %s" % name


def run_gpu(lay, budgets, pool_kernel=7, pool=B.SLKV_POOL_MAX, token_major=False):
    """token_major: K is uploaded as [T][Hkv][d] and V as [T][Hkv][d + 24] (padded rows, so V's
    strides differ from K's; + 32 for one-byte elements) instead of head-major contiguous [Hkv][T][d]."""
    import torch
    ks = vs = None
    k_host, v_host = lay.k, lay.v
    if token_major:
        pad = 32 if lay.dtype == "bf16_kv8" else 24        # strides are multiples of 16 bytes
        ks = (lay.Hkv * lay.d, lay.d)
        vs = (lay.Hkv * (lay.d + pad), lay.d + pad)
        k_host = np.ascontiguousarray(np.transpose(lay.k, (1, 0, 2)))
        v_host = np.full((lay.v.shape[1], lay.Hkv, lay.d + pad), {"bf16": 0x7F7F, "f16": 6e4, "bf16_kv8": 0x7E, "f32": 1e30}[lay.dtype], dtype=lay.v.dtype)
        v_host[:, :, :lay.d] = np.transpose(lay.v, (1, 0, 2))
    call = api.LayerCall(lay.dtype, lay.B, lay.Hq, lay.Hkv, lay.d, lay.w, lay.cu_seqlens, budgets,
                         pool_kernel, pool, debug_scores=True, k_strides=ks, v_strides=vs)
    guard = Guarded(call)
    q = api.to_device(lay.qwin, lay.dtype)
    k = api.to_device(k_host, lay.dtype)
    v = api.to_device(v_host, lay.dtype)
    call.run(q, k, v)
    torch.cuda.synchronize()
    guard.check()
    return dict(call=call, offsets=call.out_offsets.cpu().numpy(), kept=call.kept_idx.cpu().numpy(),
                k_out=api.to_host(call.k_out), v_out=api.to_host(call.v_out),
                importance=call.importance.cpu().numpy(), pooled=call.pooled.cpu().numpy())


def compare_layer(lay, budgets, gpu, pool_kernel=7, pool=B.SLKV_POOL_MAX, ref=None):
    """Element-by-element comparison of one layer's GPU result with the oracle.

    Returns a report dict: segments, exact (kept set identical), tolerant (differs only at
    positions whose score is within tolerance of the k-th score), max_rel (importance), diffs."""
    eps = TOL[lay.dtype]
    if ref is None:
        ref = oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, budgets, lay.w, pool_kernel, pool)
    host_offs, total = B.slkv_compacted_sizes(gpu["call"].layer)
    assert np.array_equal(ref["out_offsets"], host_offs), "host offsets differ from the oracle"
    assert np.array_equal(ref["out_offsets"], gpu["offsets"]), "device offsets differ from the oracle"
    G = lay.Hq // lay.Hkv
    rep = dict(segments=0, ranked=0, exact=0, tolerant=0, max_rel=0.0, diffs=[])
    for b in range(lay.B):
        t0, t1 = int(lay.cu_seqlens[b]), int(lay.cu_seqlens[b + 1])
        n = t1 - t0
        for h in range(lay.Hkv):
            s = b * lay.Hkv + h
            seg = ref["segments"][s]
            o0, o1 = int(ref["out_offsets"][s]), int(ref["out_offsets"][s + 1])
            got = gpu["kept"][o0:o1].astype(np.int64)
            rep["segments"] += 1
            # whatever was selected, the gathered rows must be bit copies of those input rows
            assert got.min(initial=0) >= 0 and got.max(initial=0) < max(n, 1)
            assert np.array_equal(gpu["k_out"][o0:o1], lay.k[h, t0 + got]), "K gather mismatch seg %d" % s
            assert np.array_equal(gpu["v_out"][o0:o1], lay.v[h, t0 + got]), "V gather mismatch seg %d" % s
            want = seg["kept_idx"]
            if seg["pooled"] is None or seg["k"] == 0:
                assert np.array_equal(got, want), "unranked segment %d differs" % s
                rep["exact"] += 1
                continue
            rep["ranked"] += 1
            m, kk = n - lay.w, seg["k"]
            so = lay.Hkv * t0 + h * n
            for name, refv in (("importance", seg["importance"]), ("pooled", seg["pooled"])):
                g = gpu[name][so:so + m].astype(np.float64)
                floor = lay.w * G / m * 1e-3
                rel = np.abs(g - refv) / np.maximum(np.abs(refv), floor)
                rep["max_rel"] = max(rep["max_rel"], float(rel.max()))
                assert rel.max() <= eps, "%s of segment %d off by %.3g (tolerance %.3g)" % (name, s, rel.max(), eps)
            assert np.array_equal(got[kk:], want[kk:]), "window of segment %d differs" % s
            assert (np.diff(got[:kk]) > 0).all(), "history of segment %d not ascending" % s
            if np.array_equal(got, want):
                rep["exact"] += 1
                continue
            # tolerance protocol: same size, holds every sure-in position, no sure-out position
            tau = seg["tau"]
            pooled = seg["pooled"]
            sure_in = set(np.nonzero(pooled > tau * (1 + eps))[0].tolist())
            sure_out = set(np.nonzero(pooled < tau * (1 - eps))[0].tolist())
            gset = set(got[:kk].tolist())
            assert len(gset) == kk
            assert sure_in <= gset, "segment %d misses a clearly-in position" % s
            assert not (gset & sure_out), "segment %d holds a clearly-out position" % s
            rep["tolerant"] += 1
            rep["diffs"].append((s, sorted(gset ^ set(want[:kk].tolist()))))
    return rep


def run_gpu_ragged(rc, budgets, pool_kernel=7, pool=B.SLKV_POOL_MAX, positions=True):
    import torch
    call = api.RaggedCall(rc.dtype, rc.B, rc.Hq, rc.Hkv, rc.d, rc.w, rc.in_offsets, budgets, pool_kernel, pool,
                          debug_scores=True, positions=positions)
    guard = Guarded(call)
    q = api.to_device(rc.qwin, rc.dtype)
    k = api.to_device(rc.k_rows, rc.dtype)
    v = api.to_device(rc.v_rows, rc.dtype)
    pos = torch.from_numpy(rc.pos_in).cuda() if positions else None
    call.run(q, k, v, pos)
    torch.cuda.synchronize()
    guard.check()
    return dict(call=call, offsets=call.out_offsets.cpu().numpy(), kept=call.kept_idx.cpu().numpy(),
                k_out=api.to_host(call.k_out), v_out=api.to_host(call.v_out),
                pos_out=call.pos_out.cpu().numpy() if positions else None,
                importance=call.importance.cpu().numpy(), pooled=call.pooled.cpu().numpy())


def compare_ragged(rc, budgets, gpu, pool_kernel=7, pool=B.SLKV_POOL_MAX):
    """As compare_layer, for slkv_recompress_layer against oracle.recompress_layer."""
    eps = TOL[rc.dtype]
    ref = oracle.recompress_layer(rc.qwin, rc.k_rows, rc.v_rows, rc.in_offsets, budgets, rc.w, pool_kernel, pool,
                                  pos_in=rc.pos_in)
    host_offs, total = B.slkv_recompress_sizes(gpu["call"].rag)
    assert np.array_equal(ref["out_offsets"], host_offs), "host offsets differ from the oracle"
    assert np.array_equal(ref["out_offsets"], gpu["offsets"]), "device offsets differ from the oracle"
    G = rc.Hq // rc.Hkv
    rep = dict(segments=0, ranked=0, exact=0, tolerant=0, max_rel=0.0)
    for s in range(rc.B * rc.Hkv):
        r0, r1 = int(rc.in_offsets[s]), int(rc.in_offsets[s + 1])
        n = r1 - r0
        seg = ref["segments"][s]
        o0, o1 = int(ref["out_offsets"][s]), int(ref["out_offsets"][s + 1])
        got = gpu["kept"][o0:o1].astype(np.int64)
        rep["segments"] += 1
        assert got.min(initial=0) >= 0 and got.max(initial=0) < max(n, 1)
        assert np.array_equal(gpu["k_out"][o0:o1], rc.k_rows[r0 + got]), "K gather mismatch seg %d" % s
        assert np.array_equal(gpu["v_out"][o0:o1], rc.v_rows[r0 + got]), "V gather mismatch seg %d" % s
        if gpu["pos_out"] is not None:
            assert np.array_equal(gpu["pos_out"][o0:o1], rc.pos_in[r0 + got]), "positions mismatch seg %d" % s
        want = seg["kept_idx"]
        if seg["pooled"] is None or seg["k"] == 0:
            assert np.array_equal(got, want), "unranked segment %d differs" % s
            rep["exact"] += 1
            continue
        rep["ranked"] += 1
        m, kk = n - rc.w, seg["k"]
        so = r0 - int(rc.in_offsets[0])
        for name, refv in (("importance", seg["importance"]), ("pooled", seg["pooled"])):
            g = gpu[name][so:so + m].astype(np.float64)
            floor = rc.w * G / m * 1e-3
            rel = np.abs(g - refv) / np.maximum(np.abs(refv), floor)
            rep["max_rel"] = max(rep["max_rel"], float(rel.max()))
            assert rel.max() <= eps, "%s of segment %d off by %.3g (tolerance %.3g)" % (name, s, rel.max(), eps)
        assert np.array_equal(got[kk:], want[kk:]), "window of segment %d differs" % s
        assert (np.diff(got[:kk]) > 0).all(), "history of segment %d not ascending" % s
        if np.array_equal(got, want):
            rep["exact"] += 1
            continue
        tau, pooled = seg["tau"], seg["pooled"]
        sure_in = set(np.nonzero(pooled > tau * (1 + eps))[0].tolist())
        sure_out = set(np.nonzero(pooled < tau * (1 - eps))[0].tolist())
        gset = set(got[:kk].tolist())
        assert len(gset) == kk
        assert sure_in <= gset, "segment %d misses a clearly-in position" % s
        assert not (gset & sure_out), "segment %d holds a clearly-out position" % s
        rep["tolerant"] += 1
    return rep
