#!/usr/bin/env python3
"""Benchmark of the SurfaceLogicKV prefill KV-compression pass on one MI355X.

A step is one slkv_compress_layer call (scoring, softmax importance, pooling, top-k, gather;
budgets precomputed with slkv_allocate_budgets) over one layer of the 32-layer
Llama-3-8B-shaped prefill: bf16, 32 query / 8 KV heads, head_dim 128, prefix 32768, window 64,
average budget 256 per KV head (fixed 16), INF_sc map with 2% spikes.  The timed loop cycles
through distinct layers (4 GiB of K/V, far above the 256 MB Infinity Cache), inputs resident
in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers 32] [--no-stage1]
"""

import argparse
import concurrent.futures as cf
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch of the dominant kernel (the statistics pass): a counter reading (rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this same command), not something this script can measure.  It is read
# from the table of the committed summary, so that it cannot go stale against it.
PROFILE_SUMMARY = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                               "compress_layer_c3_avg256_rocprofv3.md")


def measured_traffic_bytes(path=PROFILE_SUMMARY):
    """FETCH (scaled, KiB) + WRITE (KiB) of the pass-1 row of the summary's traffic table, in bytes; None if absent."""
    try:
        with open(path) as f:
            for line in f:
                cells = [c.strip() for c in line.split("|")]
                # | kernel | FETCH_SIZE | x 2.0 -> KiB read | WRITE_SIZE -> KiB written |
                if len(cells) >= 6 and cells[1].startswith("score_bf16_kernel<128,2,4,1") and "MiB" in cells[3]:
                    return (float(cells[3].split()[0]) + float(cells[4])) * 1024.0
    except (OSError, ValueError):
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--layers", type=int, default=32, help="distinct layers resident in HBM")
    ap.add_argument("--avg", type=int, default=256, help="average budget per KV head (64, 256 or 1024)")
    ap.add_argument("--no-stage1", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-recompress", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the other budgets of the sweep")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the timing of the parity configurations c1, c2 (32 rotating input copies) and c5 (one 1.2 GiB call)")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay leg")
    ap.add_argument("--no-streams", action="store_true", help="skip the two-stream leg")
    ap.add_argument("--no-peaks", action="store_true", help="skip the on-box copy / GEMM rates printed beside the datasheet peaks")
    ap.add_argument("--cpu-layers", type=int, default=32, help="layers the CPU oracle is timed on")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 256 MiB device copy (reference for the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2508_15806_amd import api, binding as B, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.lib()                                            # fail loudly when the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)

    NL = args.layers
    Hq, Hkv, d, w, n = 32, 8, 128, 64, 32768
    G = Hq // Hkv
    inf = wl.config3_inf()
    budgets = B.slkv_allocate_budgets(inf, Hkv, args.avg, 16)

    t0 = time.time()
    workers = max(1, min(16, len(os.sched_getaffinity(0))))
    with cf.ThreadPoolExecutor(workers) as ex:
        layers = list(ex.map(lambda l: wl.config3_layer(l, n), range(NL)))
    gen_s = time.time() - t0

    calls, dq, dk, dv = [], [], [], []
    for l, lay in enumerate(layers):
        calls.append(api.LayerCall("bf16", 1, Hq, Hkv, d, w, lay.cu_seqlens, budgets[l % budgets.shape[0]]))
        dq.append(api.to_device(lay.qwin, "bf16"))
        dk.append(api.to_device(lay.k, "bf16"))
        dv.append(api.to_device(lay.v, "bf16"))
    torch.cuda.synchronize()

    def step(i):
        l = i % NL
        calls[l].run(dq[l], dk[l], dv[l])

    # per-step algorithmic work
    def layer_work(l):
        bud = budgets[l % budgets.shape[0]]
        ranked = [h for h in range(Hkv) if n > bud[h] > w]
        m = n - w
        kept = int(calls[l].total_kept)
        flops = 2.0 * G * w * d * m * len(ranked)                  # one scoring pass (Eq. 7)
        byts = (len(ranked) * m * d * 2                            # K once
                + Hq * w * d * 2                                   # window queries
                + len(ranked) * m * 4 * 2                          # importance written + read
                + kept * 4                                         # kept indices
                + kept * d * 2 * 2 * 2)                            # K and V rows read + written
        big_rows = int(sum(int(c) for c in np.diff(calls[l].offsets) if c > 256))   # rows the gather launch copies
        return flops, byts, kept, len(ranked), big_rows

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    ev1.record()
    torch.cuda.synchronize()
    ms_total = ev0.elapsed_time(ev1)
    ms_step = ms_total / args.steps
    tokens_per_s = n / (ms_step * 1e-3)

    # per-step latency distribution: one event pair per step (each pair adds its own record cost)
    nlat = min(args.steps, 128)
    lat_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nlat)]
    for i in range(nlat):
        lat_ev[i][0].record()
        step(args.warmup + i)
        lat_ev[i][1].record()
    torch.cuda.synchronize()
    lat = np.array([a_.elapsed_time(b_) for a_, b_ in lat_ev])

    work = [layer_work((args.warmup + i) % NL) for i in range(args.steps)]
    flops_step = float(np.mean([x[0] for x in work]))
    bytes_step = float(np.mean([x[1] for x in work]))

    # same loop again; every kernel launch carries its own start / stop events (the kernel's
    # execution time, what a rocprofv3 kernel trace reports as its duration)
    nrec = args.steps * 8
    B.slkv_profile_begin(nrec)
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    recs = B.slkv_profile_end(nrec)
    per_kernel = {}
    for name, ms in recs:
        per_kernel.setdefault(name, []).append(ms)
    kernel_ms = {k: float(np.mean(v)) for k, v in per_kernel.items()}
    kernel_launches = {k: len(v) / args.steps for k, v in per_kernel.items()}
    dom = max(("score_stats", "score_accum"), key=lambda k: kernel_ms.get(k, 0.0))
    # launches of the scoring kernels only happen on layers with ranked heads
    ranked_flops = [x[0] for x in work if x[3] > 0]
    flops_launch = float(np.mean(ranked_flops)) if ranked_flops else 0.0
    dom_ms = kernel_ms.get(dom, float("nan"))
    achieved_tflops = flops_launch / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    traffic = measured_traffic_bytes()
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved_tflops, 2),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": traffic, "avg_ms": round(dom_ms, 5),
                "timing": "start/stop events carried by each launch of the kernel (hipExtLaunchKernelGGL), mean over the timed steps",
                "flops_per_launch": flops_launch,
                # the same launch against the HBM roof (K of the ranked heads read once per pass)
                "hbm_GBs": round(traffic / (dom_ms * 1e-3) / 1e9, 1) if traffic and dom_ms > 0 else None,
                "hbm_frac": round(traffic / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if traffic and dom_ms > 0 else None}

    out = {
        "metric": "prefix KV tokens compressed/sec per layer (1 GPU)",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c3: 32-layer Llama-3-8B-shaped prefill compression, one layer per step, "
                               "32q/8kv heads, head_dim 128, prefix 32768, window 64, pool max-7, "
                               "avg budget %d (fixed 16)" % args.avg,
                   "distinct_layers": NL, "avg_budget": args.avg, "input_gen_s": round(gen_s, 1)},
        "roofline": roofline,
        "layer": {"algorithmic_bytes": bytes_step, "hbm_GBs": round(bytes_step / (ms_step * 1e-3) / 1e9, 1),
                  "hbm_frac": round(bytes_step / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                  "one_pass_TFLOPs": round(flops_step / (ms_step * 1e-3) / 1e12, 2),
                  "step_ms_event_pairs": {"median": round(float(np.median(lat)), 5),
                                          "p10": round(float(np.percentile(lat, 10)), 5),
                                          "p90": round(float(np.percentile(lat, 90)), 5), "n": int(nlat)},
                  "kernel_ms": {k: round(v, 5) for k, v in kernel_ms.items()},
                  # the HBM-bound kernels against the chip peak: 4 B per ranked history key for the selection,
                  # 1 KiB (K and V row, read + written) per row of the segments the gather launch copies
                  "select_GBs": round(4.0 * (n - w) * float(np.mean([x[3] for x in work])) / (kernel_ms.get("select", float("nan")) * 1e-3) / 1e9, 1),
                  "gather_GBs": round(float(np.mean([x[4] for x in work if x[4] > 0] or [0.0])) * d * 2 * 2 * 2 / (kernel_ms.get("gather", float("nan")) * 1e-3) / 1e9, 1),
                  "kernel_launches_per_step": kernel_launches,
                  "kernel_sum_ms": round(sum(kernel_ms[k] * kernel_launches[k] for k in kernel_ms), 5)},
    }

    if args.calibration_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                  # 256 MiB read + 256 MiB written
        torch.cuda.synchronize()
        del src, dst

    # The same steps replayed from one HIP graph (every layer's call captured once, in order): what a
    # serving loop that cannot afford the host-side launch path would run.
    if not args.no_graph:
        gs = torch.cuda.Stream()
        gs.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(gs):
            for l in range(NL):
                calls[l].run(dq[l], dk[l], dv[l])
        torch.cuda.current_stream().wait_stream(gs)
        torch.cuda.synchronize()
        B.slkv_init()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=gs):
            for l in range(NL):
                calls[l].run(dq[l], dk[l], dv[l])
        graph.replay()
        torch.cuda.synchronize()
        reps = max(1, args.steps // NL)
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(reps):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        gms = g0.elapsed_time(g1) / (reps * NL)
        out["graph_replay"] = {"ms_per_step": round(gms, 5), "tokens_per_s": round(n / (gms * 1e-3), 1),
                               "steps": reps * NL, "graph": "%d layer calls captured into one HIP graph" % NL}
        del graph

    # The same steps with the layers dealt to two streams in turn (default priority both): layers are
    # independent of each other, and the selection's 8 workgroups leave most of the chip to the
    # scoring pass of the next layer.  Reported beside the headline, never as it.
    if not args.no_streams:
        st = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        def dealt(k):
            for i in range(k):
                l = i % NL
                with torch.cuda.stream(st[l & 1]):      # a layer always runs on the same stream
                    calls[l].run(dq[l], dk[l], dv[l])
        dealt(args.warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dealt(args.steps)
        torch.cuda.synchronize()
        tms = (time.perf_counter() - t0) * 1e3 / args.steps
        out["two_streams"] = {"ms_per_step": round(tms, 5), "tokens_per_s": round(n / (tms * 1e-3), 1), "steps": args.steps,
                              "note": "independent layers alternate between two streams; not the headline"}

    # What this machine sustains, printed beside the datasheet peaks the fractions are taken against
    if not args.no_peaks:
        src = torch.empty(128 << 20, dtype=torch.float32, device=dev).normal_()      # 512 MiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        for _ in range(5):
            dst.copy_(src)
        p1.record()
        torch.cuda.synchronize()
        copy_gbs = 5 * 2 * src.numel() * 4 / (p0.elapsed_time(p1) * 1e-3) / 1e9
        del src, dst
        a_ = torch.randn(8192, 8192, dtype=torch.bfloat16, device=dev)
        b_ = torch.randn(8192, 8192, dtype=torch.bfloat16, device=dev)
        torch.mm(a_, b_)
        torch.cuda.synchronize()
        p0.record()
        for _ in range(5):
            torch.mm(a_, b_)
        p1.record()
        torch.cuda.synchronize()
        gemm_tflops = 5 * 2 * 8192.0 ** 3 / (p0.elapsed_time(p1) * 1e-3) / 1e12
        del a_, b_
        out["peaks"] = {"hbm_datasheet_GBs": HBM_PEAK_GBS, "mfma_bf16_datasheet_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
                        "measured_copy_GBs": round(copy_gbs, 1),
                        "measured_bf16_gemm_TFLOPs": round(gemm_tflops, 1),
                        "note": "measured: 512 MiB device copy (read + write bytes) and an 8192^3 bf16 torch.mm on this box"}

    # other budgets of the sweep (same inputs, shorter loops)
    sweep = {}
    sweep_calls = {}
    for avg in wl.C3_BUDGETS:
        if avg == args.avg or args.no_sweep:
            continue
        bud = B.slkv_allocate_budgets(inf, Hkv, avg, 16)
        cs = [api.LayerCall("bf16", 1, Hq, Hkv, d, w, layers[l].cu_seqlens, bud[l % 32]) for l in range(NL)]
        for i in range(NL):
            cs[i % NL].run(dq[i % NL], dk[i % NL], dv[i % NL])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(NL, args.steps // 2)
        e0.record()
        for i in range(reps):
            cs[i % NL].run(dq[i % NL], dk[i % NL], dv[i % NL])
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        sweep["avg%d" % avg] = {"ms_per_step": round(ms, 5), "tokens_per_s": round(n / (ms * 1e-3), 1)}
        sweep_calls[avg] = (bud, cs)
    out["budget_sweep"] = sweep

    if not args.no_other_configs:
        def time_config(lay, bud, copies, reps):
            cs = [api.LayerCall(lay.dtype, lay.B, lay.Hq, lay.Hkv, lay.d, lay.w, lay.cu_seqlens, bud) for _ in range(copies)]
            qs = [api.to_device(lay.qwin, lay.dtype) for _ in range(copies)]
            ks = [api.to_device(lay.k, lay.dtype) for _ in range(copies)]
            vs = [api.to_device(lay.v, lay.dtype) for _ in range(copies)]
            for i in range(copies):
                cs[i].run(qs[i], ks[i], vs[i])
            torch.cuda.synchronize()
            a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a_.record()
            for r in range(reps):
                cs[r % copies].run(qs[r % copies], ks[r % copies], vs[r % copies])
            b_.record()
            torch.cuda.synchronize()
            ms_ = a_.elapsed_time(b_) / reps
            toks = int(lay.cu_seqlens[-1])
            return {"ms_per_call": round(ms_, 5), "tokens_per_s": round(toks / (ms_ * 1e-3), 1), "input_copies": copies}
        other = {}
        lay = wl.config1()
        other["c1"] = time_config(lay, B.slkv_allocate_budgets(lay.meta["inf"], lay.Hkv, lay.meta["avg"], lay.meta["fixed"])[0], 32, 128)
        lay = wl.config2()
        other["c2"] = time_config(lay, B.slkv_allocate_budgets(lay.meta["inf"], lay.Hkv, lay.meta["avg"], lay.meta["fixed"])[0], 32, 128)
        lay = wl.config5()
        other["c5"] = time_config(lay, B.slkv_allocate_budgets(inf, Hkv, 512, 64)[wl.config5_layer_row(inf)], 1, 10)
        # the headline workload with keys and values stored as E4M3 bytes (8 of its layers, re-encoded on the device)
        NK = min(8, NL)
        k8 = [dk[l].float().to(torch.float8_e4m3fn).view(torch.uint8) for l in range(NK)]
        v8 = [dv[l].float().to(torch.float8_e4m3fn).view(torch.uint8) for l in range(NK)]
        c8 = [api.LayerCall("bf16_kv8", 1, Hq, Hkv, d, w, layers[l].cu_seqlens, budgets[l % budgets.shape[0]]) for l in range(NK)]
        for r in range(2 * NK):
            c8[r % NK].run(dq[r % NK], k8[r % NK], v8[r % NK])
        torch.cuda.synchronize()
        a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a_.record()
        for r in range(128):
            c8[r % NK].run(dq[r % NK], k8[r % NK], v8[r % NK])
        b_.record()
        torch.cuda.synchronize()
        ms8 = a_.elapsed_time(b_) / 128
        other["c3_kv_e4m3"] = {"ms_per_call": round(ms8, 5), "tokens_per_s": round(n / (ms8 * 1e-3), 1), "input_copies": NK,
                               "note": "bf16 queries, keys and values as OCP E4M3 bytes (not the headline dtype)"}
        del k8, v8, c8
        out["other_configs"] = other
        del lay

    # Decode-time re-compression of a grown ragged cache (c6): 32 sequences x 8 KV heads
    if not args.no_recompress:
        row = wl.config5_layer_row(inf)
        bud6 = budgets[row]
        kept_after_prefill = B.slkv_compacted_sizes(B.Layer(B.SLKV_BF16, 1, Hq, Hkv, d, w, [0, n], bud6,
                                                            (d, n * d), (d, n * d)))[0]
        lens = [int(x) + 128 for x in np.diff(kept_after_prefill)]
        rc = wl.config6(lens, batch=32)
        call6 = api.RaggedCall("bf16", rc.B, rc.Hq, rc.Hkv, rc.d, rc.w, rc.in_offsets, bud6)
        q6, k6, v6 = api.to_device(rc.qwin, "bf16"), api.to_device(rc.k_rows, "bf16"), api.to_device(rc.v_rows, "bf16")
        p6 = torch.from_numpy(rc.pos_in).to(dev)
        for _ in range(8):
            call6.run(q6, k6, v6, p6)
        torch.cuda.synchronize()
        reps = 64
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call6.run(q6, k6, v6, p6)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        rows_in = int(rc.in_offsets[-1])
        out["recompress"] = {"workload": "c6: 32 sequences x 8 KV heads, cache = kept rows of avg-256 budgets + 128 new tokens, "
                                         "window 64, bf16 (warm cache: one input set)",
                             "segments": int(rc.B * rc.Hkv), "rows_in": rows_in, "rows_out": int(call6.total_kept),
                             "ms_per_call": round(ms, 5), "cached_rows_per_s": round(rows_in / (ms * 1e-3), 1)}
        del q6, k6, v6, call6

    # Stage 1 (Algorithm 1) on the 32 x 32 heads x 16 steps x 16384 attention rows (1 GiB)
    if not args.no_stage1:
        nr = wl.config4()
        rows = torch.from_numpy(nr.rows).to(dev)
        acc, sc = api.score_heads(rows, nr.needle_start, nr.needle_len, nr.topk)
        torch.cuda.synchronize()
        reps = 5
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            api.score_heads(rows, nr.needle_start, nr.needle_len, nr.topk, acc)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        B.slkv_profile_begin(reps * 2)                  # same calls again with an event pair per kernel
        for _ in range(reps):
            api.score_heads(rows, nr.needle_start, nr.needle_len, nr.topk, acc)
        torch.cuda.synchronize()
        recs1 = B.slkv_profile_end(reps * 2)
        rc_ms = float(np.mean([m_ for k_, m_ in recs1 if k_ == "row_cells"]))
        nbytes = rows.numel() * 4
        # bandwidth over the whole call (row kernel + per-head reduction + launch gaps): the conservative figure
        out["stage1"] = {"workload": "c4: 32x32 heads x 16 decode rows x 16384 weights fp32",
                         "ms_per_call": round(ms, 4), "rows_per_s": round(rows.shape[0] * rows.shape[1] * rows.shape[2] / (ms * 1e-3), 1),
                         "row_cells_ms": round(rc_ms, 4), "hbm_GBs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                         "hbm_frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del rows

    # Stage 1 straight from decode queries and context keys (same shape; the attention rows are never in memory)
    if not args.no_stage1:
        x = wl.config4_qk()
        q4, k4 = api.to_device(x.q, "bf16"), api.to_device(x.k, "bf16")
        acc4, _ = api.score_heads_qk(q4, k4, x.needle_start, x.needle_len, x.topk)
        torch.cuda.synchronize()
        reps = 5
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            api.score_heads_qk(q4, k4, x.needle_start, x.needle_len, x.topk, acc4)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        kbytes = k4.numel() * 2
        out["stage1_from_qk"] = {"workload": "the same 32x32 heads x 16 decode rows over 16384 keys, rows computed on chip from bf16 Q and K",
                                 "ms_per_call": round(ms, 4), "rows_per_s": round(32 * 32 * 16 / (ms * 1e-3), 1),
                                 "key_bytes": kbytes, "key_GBs": round(kbytes / (ms * 1e-3) / 1e9, 1),
                                 "hbm_frac_keys_once": round(kbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del q4, k4, x

    # CPU baseline: the float64 oracle, as it stands, on a bounded sample of the same workload,
    # also used as the parity check of what the GPU just produced.
    if not args.no_cpu:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        ncpu = min(args.cpu_layers, NL)
        t0 = time.time()
        refs, caches = [], []
        for l in range(ncpu):
            lay = layers[l]
            caches.append({})
            refs.append(oracle.compress_layer(lay.qwin, lay.k, lay.v, lay.cu_seqlens, budgets[l], w, 7, score_cache=caches[l]))
        cpu_s = time.time() - t0
        cpu_model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                for line in f:
                    if line.startswith("model name"):
                        cpu_model = line.split(":", 1)[1].strip()
                        break
        except OSError:
            pass
        out["cpu_baseline"] = {"value": round(ncpu * n / cpu_s, 1), "unit": "tokens/s", "cores": int(cores),
                               "kind": "oracle", "cpu": cpu_model,
                               "sample": "%d of the %d layers of the same workload, float64 numpy" % (ncpu, NL)}

        # every timed output against the oracle: the main budget and the budgets of the sweep
        def check(avg, bud_map, call_list, ref_list):
            exact = total = ranked = 0
            for l in range(ncpu):
                call_list[l].run(dq[l], dk[l], dv[l])
                torch.cuda.synchronize()
                kept = call_list[l].kept_idx.cpu().numpy()
                offs = ref_list[l]["out_offsets"]
                same_rows = (np.array_equal(api.to_host(call_list[l].k_out)[:offs[-1]], ref_list[l]["k_out"])
                             and np.array_equal(api.to_host(call_list[l].v_out)[:offs[-1]], ref_list[l]["v_out"]))
                for s_ in range(Hkv):
                    total += 1
                    ranked += int(ref_list[l]["segments"][s_]["pooled"] is not None and ref_list[l]["segments"][s_]["k"] > 0)
                    exact += int(same_rows and np.array_equal(kept[offs[s_]:offs[s_ + 1]], ref_list[l]["segments"][s_]["kept_idx"]))
            return {"avg_budget": avg, "segments_checked": total, "ranked": ranked, "kept_sets_and_rows_identical": exact}
        parity = [check(args.avg, budgets, calls, refs)]
        for avg, (bud, cs) in sorted(sweep_calls.items()):
            refs2 = [oracle.compress_layer(layers[l].qwin, layers[l].k, layers[l].v, layers[l].cu_seqlens, bud[l], w, 7,
                                           score_cache=caches[l]) for l in range(ncpu)]
            parity.append(check(avg, bud, cs, refs2))
        out["parity"] = parity
    print(json.dumps(out))


if __name__ == "__main__":
    main()
