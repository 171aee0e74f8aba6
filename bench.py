#!/usr/bin/env python3
"""Benchmark of the CalibQuant hot path on one MI355X.

One "step" is one cq_decode_attn call (logits from the packed 1-bit cache, calibration,
joint softmax with the fp16 text tail, weighted value sum) over one batch of a synthetic
InternVL-shaped cache that is already resident in HBM.  The quantizer (cq_quantize_kv)
that produces the cache is timed in the same run and reported under "quantizer".

Prints ONE JSON line.  `value` = KV tokens attended per second = B*(n_vis+n_text)/t.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth


def algorithmic_bytes(w, bits, k_group, v_group):
    """Bytes the method has to move for one decode call (workspace traffic is not counted).

    Per visual token per KV head: K codes + K (scale fp32 + min fp16)/k_group tokens per channel
    + V codes + one (scale, min) pair per v_group channels; per text token per KV head 2*d fp16
    for K and V; plus q and out.
    """
    d = w.head_dim
    per_vis = 2 * d * bits / 8 + 6.0 * d / k_group + 6.0 * d / v_group
    per_text = 2 * d * 2
    rows = w.batch * w.n_kv_heads
    qo = 2 * w.batch * w.n_q_heads * d * 2
    return rows * (w.n_vis * per_vis + w.n_text * per_text) + qo, per_vis, per_text


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="index into the workload list")
    ap.add_argument("--bits", type=int, default=1)
    ap.add_argument("--group", type=int, default=128,
                    help="tokens per key group (32, 64, 128); 0 = statistics over the whole "
                         "sequence, one pair per channel (the paper's scheme as printed)")
    ap.add_argument("--v-axis", choices=["token", "channel"], default="token",
                    help="value statistics: per token (the benchmark's layout) or per channel over "
                         "groups of tokens (the paper's own choice)")
    ap.add_argument("--path", choices=["auto", "generic", "tuned"], default="auto")
    ap.add_argument("--launch", choices=["graph", "eager"], default="graph",
                    help="how the timed steps are launched: replay of one HIP graph holding all "
                         "of them (a serving loop's way), or one call per step from Python")
    ap.add_argument("--chunks", type=int, default=0,
                    help="at least this many chunks per row of the tuned decode (0 = the library's "
                         "own choice): forces the split-row kernels on rows that one workgroup could own")
    ap.add_argument("--tau-search", action="store_true",
                    help="also run and time the grid search of the calibration parameters")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fp16-baseline", action="store_true")
    ap.add_argument("--batch", type=int, default=0, help="override the batch (debugging only)")
    ap.add_argument("--n-vis", type=int, default=0, help="override the visual tokens (debugging only)")
    ap.add_argument("--q-heads", type=int, default=0, help="override the query heads (debugging only)")
    ap.add_argument("--n-text", type=int, default=-1, help="override the text tokens (debugging only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2502_14882_amd import binding as cq
    from paper_2502_14882_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    cq.lib()    # fail loudly if libcq.so is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cq.cq_bench_set_kernel_path({"auto": cq.CQ_PATH_AUTO, "generic": cq.CQ_PATH_GENERIC,
                           "tuned": cq.CQ_PATH_TUNED}[args.path])

    cq.cq_bench_set_decode_chunks(args.chunks)

    w = synth.WORKLOADS[args.config]
    if args.batch:
        w = w.replace(batch=args.batch)
    if args.n_vis:
        w = w.replace(n_vis=args.n_vis)
    if args.q_heads:
        w = w.replace(n_q_heads=args.q_heads)
    if args.n_text >= 0:
        w = w.replace(n_text=args.n_text)

    def timed(fn, reps):
        """Median device time of fn over reps (HIP events on the current stream), in ms."""
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ts.sort()
        return ts[len(ts) // 2], ts[0]

    if w.n_text == 0 and w.n_q_heads == w.n_kv_heads:
        # the quantizer-only workload: sweep group size and bit width, report GB/s read+written
        x = synth.make_inputs(w, dev, parts=("k", "v"))
        rows = w.batch * w.n_kv_heads
        sweep = []
        for bits in (1, 2):
            for group in (32, 64, 128):
                lay = cq.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_vis, bits,
                                     cq.CQ_AXIS_CHANNEL, cq.CQ_AXIS_TOKEN, group, group)
                k_q = cq.alloc_qtensor(lay, lay.k_axis, group, dev)
                v_q = cq.alloc_qtensor(lay, lay.v_axis, group, dev)
                cq.cq_quantize_kv(lay, x["k"], x["v"], k_q, v_q)
                torch.cuda.synchronize()
                med, mn = timed(lambda: cq.cq_quantize_kv(lay, x["k"], x["v"], k_q, v_q),
                                max(5, args.steps // 10))
                nbytes = rows * w.n_vis * (2 * w.head_dim * 2 + 2 * w.head_dim * bits / 8
                                           + 6.0 * w.head_dim / group * 2)
                # the same reads and writes without the arithmetic: what this traffic costs on this machine
                n_tiles = rows * w.n_vis // 128
                cb, mb = 2048 * bits, 768 * 128 // group
                sc_c = torch.empty(n_tiles * cb, dtype=torch.uint8, device=dev)
                sc_m = torch.empty(n_tiles * mb, dtype=torch.uint8, device=dev)
                tr_med, _ = timed(lambda: (cq.cq_bench_tile_traffic(x["k"], sc_c, sc_m, n_tiles, cb, mb),
                                           cq.cq_bench_tile_traffic(x["v"], sc_c, sc_m, n_tiles, cb, mb)), 10)
                sweep.append({"bits": bits, "group": group, "ms": med, "min_ms": mn,
                              "bytes_read_plus_written": nbytes,
                              "GB/s": nbytes / (med * 1e-3) / 1e9,
                              "frac_of_hbm_peak": nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "same_traffic_without_arithmetic_ms": tr_med,
                              "quantizer_vs_traffic_only": tr_med / med})
                del k_q, v_q, sc_c, sc_m
        # practical ceiling: plain streaming reads of the same two input tensors
        in_bytes = x["k"].numel() * 2
        rd_ms, _ = timed(lambda: (cq.cq_bench_stream_read(x["k"], in_bytes),
                                  cq.cq_bench_stream_read(x["v"], in_bytes)), 10)
        best = [e for e in sweep if e["bits"] == 1 and e["group"] == 128][0]
        print(json.dumps({
            "metric": "quantize_kv_bytes_read_plus_written_per_s", "value": best["GB/s"],
            "unit": "GB/s", "n_gpus": 1, "steps": max(5, args.steps // 10), "warmup": 1,
            "ms_per_step": best["ms"], "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f16 in, u1/u2 codes + f32 scale + f16 min out",
            "data": "synthetic",
            "config": {"workload": "configs[%d] %s" % (args.config, w.name), "batch": w.batch,
                       "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "n_vis": w.n_vis,
                       "kernel_path": args.path},
            "roofline": {"bound": "hbm", "achieved": best["GB/s"], "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": best["frac_of_hbm_peak"], "traffic": None,
                         "kernel": "quantize_tile_kernel (keys + values launches)",
                         "stream_read_of_the_input": {
                             "ms": rd_ms, "GB/s": 2 * in_bytes / (rd_ms * 1e-3) / 1e9,
                             "frac_of_hbm_peak": 2 * in_bytes / (rd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}},
            "sweep": sweep}))
        return 0
    # --group is the key group (tokens); token-wise values keep one group per token, channel-wise
    # values use the same token group as the keys
    k_group = args.group if args.group > 0 else w.n_vis
    v_group = k_group if args.v_axis == "channel" else w.head_dim
    lay = cq.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_vis, args.bits,
                         cq.CQ_AXIS_CHANNEL,
                         cq.CQ_AXIS_CHANNEL if args.v_axis == "channel" else cq.CQ_AXIS_TOKEN,
                         k_group, v_group)
    calib = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    bytes_call, per_vis, per_text = algorithmic_bytes(w, args.bits, k_group, v_group)

    # ---- resident inputs: several independent sets so that no call finds its cache warm
    n_sets = int(min(32, max(3, math.ceil(800e6 / bytes_call))))
    sets = []
    quant_ms = []
    for i in range(n_sets):
        x = synth.make_inputs(w, dev, seed=w.seed + 7919 * i)
        k_q = cq.alloc_qtensor(lay, lay.k_axis, lay.k_group, dev)
        v_q = cq.alloc_qtensor(lay, lay.v_axis, lay.v_group, dev)
        for rep in range(2):      # first pass warms up, second is timed
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            cq.cq_quantize_kv(lay, x["k"], x["v"], k_q, v_q)
            e1.record()
            torch.cuda.synchronize()
            if rep == 1:
                quant_ms.append(e0.elapsed_time(e1))
        sets.append(dict(q=x["q"], k=k_q, v=v_q, k_text=x["k_text"], v_text=x["v_text"],
                         out=torch.empty_like(x["q"])))
        if i == 0 and not args.no_cpu_baseline:      # the oracle's inputs: set 0, whole, on the host
            host0 = {n: x[n].cpu().numpy() for n in ("k", "v", "q", "k_text", "v_text")}
        del x
    ws = torch.empty(cq.cq_decode_workspace_bytes(lay, w.n_text, calib), dtype=torch.uint8, device=dev)

    def step(i):
        s = sets[i % n_sets]
        cq.cq_decode_attn(lay, s["q"], s["k"], s["v"], s["k_text"], s["v_text"], w.n_text, calib,
                          0.0, s["out"], ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # per-step HIP events over eagerly launched steps: the spread of single launches
    n_ev = args.steps if args.launch == "eager" else min(args.steps, 100)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(n_ev)]
    t0 = time.perf_counter()
    for i in range(n_ev):
        ev[i][0].record()
        step(i)
        ev[i][1].record()
    torch.cuda.synchronize()
    eager_wall_ms = (time.perf_counter() - t0) * 1e3 / n_ev
    dev_ms = sorted(a.elapsed_time(b) for a, b in ev)
    med_ms, min_ms = dev_ms[len(dev_ms) // 2], dev_ms[0]
    eager_mean_ms = sum(dev_ms) / len(dev_ms)

    if args.launch == "graph":
        # The timed region.  A step is one cq_decode_attn call; `steps` of them are recorded once
        # into a HIP graph (the library allocates nothing and calls no blocking API per step) and
        # the graph is replayed back to back until at least MIN_TIMED launches lie between the two
        # events, whatever `steps` is: a replay costs ~0.3 ms before its first kernel, which a short
        # region would book on its few steps.  At least MIN_SETTLE launches run untimed immediately
        # before the first event, without a synchronisation in between, so that the timed replays
        # are already queued behind work in flight and the clocks have settled.
        # One recorded graph holds a whole number of K-step blocks, at least MIN_GRAPH launches:
        # between two replays the device idles for ~7 us, which short graphs would book on their
        # few steps (at K = 20 it added 0.4 us to every step).
        MIN_TIMED, MIN_SETTLE, MIN_GRAPH = 1000, 200, 250
        per_graph = args.steps * -(-MIN_GRAPH // args.steps)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(per_graph):
                step(i)
        n_timed = -(-MIN_TIMED // per_graph)
        n_settle = -(-MIN_SETTLE // per_graph)
        graph.replay()                      # untimed: instantiation and upload
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        for _ in range(n_settle):
            graph.replay()
        e0.record()
        for _ in range(n_timed):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        wall_all_ms = (time.perf_counter() - t0) * 1e3
        timed_launches = n_timed * per_graph
        mean_ms = e0.elapsed_time(e1) / timed_launches
        # host wall clock over settle + timed replays, per launch: an upper bound that also holds
        # the launch of the first replay
        wall_ms = wall_all_ms / ((n_settle + n_timed) * per_graph)
        # a replayed step must give what the eager step gives
        last = sets[(per_graph - 1) % n_sets]
        from_graph = last["out"].clone()
        step(per_graph - 1)
        torch.cuda.synchronize()
        if not torch.equal(from_graph, last["out"]):
            raise RuntimeError("graph replay and eager launch disagree")
    else:
        wall_ms, mean_ms = eager_wall_ms, eager_mean_ms
        timed_launches = n_ev

    kv_tokens = w.batch * (w.n_vis + w.n_text)
    # throughput and ms_per_step from the device time of the timed region (HIP events on the
    # launches' stream); the host's wall clock per launch is reported next to it
    value = kv_tokens / (mean_ms * 1e-3)
    achieved = bytes_call / (mean_ms * 1e-3) / 1e9

    # practical ceiling: a plain streaming read of the same number of bytes, cold each time
    probe = torch.empty(int(bytes_call) * 3 + 64, dtype=torch.uint8, device=dev)
    nb = int(bytes_call) // 16 * 16
    # launched the way the timed steps are (one graph of 30 reads over three regions in turn, replayed
    # back to back), so that it is the kernel that is timed and not the launch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for i in range(3):
            cq.cq_bench_stream_read(probe[i * nb:], nb)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    rgraph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(rgraph):
        for i in range(30):
            cq.cq_bench_stream_read(probe[(i % 3) * nb:], nb)
    rgraph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rgraph.replay()
    e0.record()
    for _ in range(10):
        rgraph.replay()
    e1.record()
    torch.cuda.synchronize()
    stream_ms = e0.elapsed_time(e1) / 300.0
    del rgraph
    # ---- 16-bit baseline in the same harness (the paper's "16-bit baseline", Sec. 4.4): the same
    # call with the whole cache left in fp16, i.e. no visual tokens and every token in the fp16
    # tail.  Same kernel family, same launch path, nothing quantized.
    fp16_baseline = None
    if not args.no_fp16_baseline:
        n_all = w.n_vis + w.n_text
        lay16 = cq.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, 0, args.bits,
                               cq.CQ_AXIS_CHANNEL, cq.CQ_AXIS_TOKEN, 128, 128)
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed + 17)
        shape16 = (w.batch, w.n_kv_heads, n_all, w.head_dim)
        sets16 = [(torch.randn(shape16, generator=gen, device=dev, dtype=torch.float16),
                   torch.randn(shape16, generator=gen, device=dev, dtype=torch.float16))
                  for _ in range(2)]
        ws16 = torch.empty(cq.cq_decode_workspace_bytes(lay16, n_all), dtype=torch.uint8, device=dev)
        none = cq.make_calib(cq.CQ_CALIB_NONE)

        def step16(i):
            k16, v16 = sets16[i % 2]
            cq.cq_decode_attn(lay16, sets[0]["q"], None, None, k16, v16, n_all, none, 0.0,
                              sets[0]["out"], ws16)

        prev_path = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
        try:
            step16(0)
            torch.cuda.synchronize()
            kernel16 = "fused_row_kernel, text path only (one launch)"
        except cq.CqError:
            cq.cq_bench_set_kernel_path(cq.CQ_PATH_AUTO)
            kernel16 = "shape-agnostic kernels (the row does not fit the tuned kernel's LDS)"
        n16 = 20 if kernel16.startswith("fused") else 3
        for i in range(2):
            step16(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n16):
            step16(i)
        e1.record()
        torch.cuda.synchronize()
        cq.cq_bench_set_kernel_path(prev_path)
        ms16 = e0.elapsed_time(e1) / n16
        bytes16 = w.batch * w.n_kv_heads * n_all * per_text + 2 * w.batch * w.n_q_heads * w.head_dim * 2
        fp16_baseline = {"ms": ms16, "kernel": kernel16, "bytes_per_call": bytes16,
                         "GB/s": bytes16 / (ms16 * 1e-3) / 1e9,
                         "frac_of_hbm_peak": bytes16 / (ms16 * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "speedup_of_quantized_cache": ms16 / mean_ms,
                         "cache_bytes_ratio": bytes16 / bytes_call}
        del sets16, ws16

    # ---- optional: the grid search of tau1, tau2 (Sec. 3.2) on the first input set
    tau_search = None
    if args.tau_search:
        xs = synth.make_inputs(w, dev, seed=w.seed)
        k_s, _ = cq.cq_quantize_kv(lay, xs["k"], xs["v"])
        del xs["v"]
        grid = (0.0, 1.0, 2.0, 3.0)
        ws_t = torch.empty(cq.cq_tau_search_workspace_bytes(lay, w.n_text, 4, 4), dtype=torch.uint8,
                           device=dev)
        kt_s = xs["k_text"] if w.n_text > 0 else None
        run = lambda: cq.cq_tau_search(lay, xs["q"], xs["k"], k_s, kt_s, w.n_text, grid, grid, 0.0, ws_t)
        mse = run()
        torch.cuda.synchronize()
        t_med, t_min = timed(run, 3)
        mse = mse.cpu().numpy()
        i1, i2 = divmod(int(mse.argmin()), 4)
        tau_search = {"ms": t_med, "grid": list(grid), "mse": [[float(v) for v in r] for r in mse],
                      "best_tau1_tau2": [grid[i1], grid[i2]], "mse_without_calibration": float(mse[0][0]),
                      "workspace_bytes": ws_t.numel(),
                      "note": "mean squared error of the attention weights against those of the exact "
                              "keys, synthetic keys; shape-agnostic logits kernels + fp64 weights"}
        del xs, k_s, ws_t

    # one plain copy of known size: the launch that byte counters (FETCH_SIZE / WRITE_SIZE) are
    # scaled with when this command runs under rocprofv3 --pmc
    cq.cq_bench_stream_copy(probe[nb:], probe, nb)
    torch.cuda.synchronize()
    del probe

    # quantizer figures (bytes read + written per call)
    rows = w.batch * w.n_kv_heads
    # a tensor with whole-sequence statistics is read twice (extrema pass, then codes)
    q_reads = (2 if k_group == w.n_vis else 1) + (2 if v_group == w.n_vis and args.v_axis == "channel" else 1)
    q_bytes = rows * w.n_vis * (q_reads * w.head_dim * 2) + rows * w.n_vis * (per_vis)
    q_ms = sorted(quant_ms)[len(quant_ms) // 2]

    # which kernel ran: forcing the tuned path fails loudly when the layout would fall back
    prev_path = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        step(0)
        torch.cuda.synchronize()
        fused = args.path != "generic"
    except cq.CqError:
        fused = False
    cq.cq_bench_set_kernel_path(prev_path)
    split = fused and ws.numel() > 256          # rows split over workgroups: the scratch says so
    streamed = split and ws.numel() > w.batch * w.n_q_heads * w.n_vis * 2
    kernel_name = ("stream_logits_kernel + stream_values_kernel + combine_kernel (all launches of one call)"
                   if streamed else
                   "fused_row_kernel, extrema pass + partial pass, + combine_kernel (all launches of one call)"
                   if split else
                   "fused_row_kernel<%d> (the call's only launch)" % (min(k_group, 128) // 16) if fused
                   else "scores_kernel + pv_kernel + combine_kernel (all launches of one call)")
    # HBM bytes per launch from hardware counters: NOT measured by this run.  The committed summary
    # of two rocprofv3 --pmc runs of this command holds the figure together with the SHA-256 of the
    # kernel source it was taken on; it is reported only while that source is unchanged.
    traffic, traffic_source = None, None
    if (fused and args.config == 2 and args.bits == 1 and args.group == 128 and not args.batch and not args.n_vis and not args.q_heads and args.n_text < 0
            and args.v_axis == "token"):
        import hashlib
        prof = os.path.join("profiles", "fused_row_kernel_configs2_hbm_traffic.txt")
        # the kernel and the device helpers it includes, hashed together in this order
        srcs = [os.path.join("paper_2502_14882_amd", "csrc", f) for f in ("decode_fused.hip", "decode_device.h")]
        src = " + ".join(srcs)
        try:
            sha_now = hashlib.sha256(b"".join(open(os.path.join(ROOT, f), "rb").read() for f in srcs)).hexdigest()[:16]
            val, sha_prof = None, None
            for line in open(os.path.join(ROOT, prof)):
                if line.startswith("fused_row_kernel_configs2_traffic_bytes_per_launch:"):
                    val = float(line.split(":")[1])
                if line.startswith("kernel_source_sha256_16:"):
                    sha_prof = line.split(":")[1].strip()
            if val is not None and sha_prof == sha_now:
                traffic = val
                traffic_source = "%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, taken on %s sha256 %s)" % (prof, src, sha_prof)
            else:
                traffic_source = "not reported: %s was taken on another version of %s" % (prof, src)
        except OSError:
            traffic_source = "not reported: no committed counter summary"

    result = {
        "metric": "decode_attention_kv_tokens_per_s",
        "value": value,
        "unit": "KV tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": mean_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u1 codes, f16 text/query, f32 accumulate" if args.bits == 1
                 else "u%d codes, f16 text/query, f32 accumulate" % args.bits,
        "data": "synthetic",
        "config": {"workload": "configs[%d] %s" % (args.config, w.name), "batch": w.batch,
                   "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "n_vis": w.n_vis, "n_text": w.n_text, "bits": args.bits,
                   "k_group": k_group, "v_group": v_group, "v_axis": args.v_axis,
                   "calib": "dynamic tau=(1,2)",
                   "kernel_path": args.path, "min_chunks": args.chunks, "input_sets": n_sets},
        "launch": args.launch,
        "timed_region": {"launches_between_events": timed_launches,
                         "note": "one graph of whole `steps`-blocks (>= 250 launches) replayed back to "
                                 "back, preceded by >= 200 untimed launches with no synchronisation "
                                 "in between"
                                 if args.launch == "graph" else "one call per step from Python",
                         "host_wall_ms_per_launch": wall_ms},
        "device_ms": {"mean_in_timed_region": mean_ms, "eager_median": med_ms, "eager_min": min_ms,
                      "eager_mean": eager_mean_ms, "eager_wall_per_step": eager_wall_ms},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": traffic_source,
                     "kernel": kernel_name,
                     "algorithmic_bytes_per_call": bytes_call,
                     "stream_read_same_bytes": {"ms": stream_ms,
                                                "GB/s": nb / (stream_ms * 1e-3) / 1e9,
                                                "frac_of_hbm_peak": nb / (stream_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                                "decode_vs_stream_read": stream_ms / mean_ms},
                     "bytes_per_visual_token_per_kv_head": per_vis,
                     "bytes_per_text_token_per_kv_head": per_text},
        "fp16_baseline": fp16_baseline,
        "tau_search": tau_search,
        "quantizer": {"ms": q_ms, "bytes_read_plus_written": q_bytes, "reads_of_k_plus_v": q_reads,
                      "GB/s": q_bytes / (q_ms * 1e-3) / 1e9,
                      "frac_of_hbm_peak": q_bytes / (q_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "tokens_per_s": rows * w.n_vis / (q_ms * 1e-3)},
        "whole_path_500_tokens": {
            "note": "one quantize + 500 decode steps, as in the paper's overall-throughput column",
            "sequences_per_s": w.batch / ((q_ms + 500 * mean_ms) * 1e-3)},
    }

    if not args.no_cpu_baseline:
        # The oracle as it stands (its C++ form: dequantize, then plain fp64 loops, rows spread over
        # the host's threads with OpenMP) on the WHOLE call of input set 0: it quantizes the fp16
        # cache itself (untimed here, reported separately), then the decode step is timed.
        from oracle import cq_oracle as O
        from oracle import cq_oracle_native as ON
        v_ax = O.AXIS_CHANNEL if args.v_axis == "channel" else O.AXIS_TOKEN
        c0 = time.perf_counter()
        kq = ON.quantize_tensor(host0["k"], args.bits, O.AXIS_CHANNEL, k_group)
        vq = ON.quantize_tensor(host0["v"], args.bits, v_ax, v_group)
        t_quant = time.perf_counter() - c0
        n_rep, t_used = 0, 0.0
        while t_used < 10.0 and n_rep < 20:
            c0 = time.perf_counter()
            ref = ON.decode_attn(host0["q"], kq, vq, host0["k_text"], host0["v_text"], w.n_text,
                                 O.CALIB_DYNAMIC, 1.0, 2.0)
            t_used += time.perf_counter() - c0
            n_rep += 1
        step(0)
        torch.cuda.synchronize()
        got = sets[0]["out"].cpu().numpy().astype(np.float64)
        result["cpu_baseline"] = {
            "value": kv_tokens * n_rep / t_used, "unit": "KV tokens/s",
            "cores": ON.max_threads(), "kind": "oracle",
            "sample": "whole call: all %d sequences of input set 0, %d repeats of the decode step, %.1f s"
                      % (w.batch, n_rep, t_used),
            "s_per_call": t_used / n_rep, "oracle_quantize_s": t_quant,
            "host_cpus": os.cpu_count(),
            "parity_rel_l2_whole_call": O.rel_l2(got, ref),
            "parity_worst_row_rel_l2": float((np.linalg.norm(got - ref, axis=-1)
                                              / np.linalg.norm(ref, axis=-1)).max())}

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
