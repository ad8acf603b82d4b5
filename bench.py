#!/usr/bin/env python3
"""Benchmark of the decode-step hybrid-head attention on one MI355X.

A *step* is the attention of one whole decode step on the Qwen3-8B-shaped 128K workload
(36 layers, 32 query / 8 KV heads, head dim 128, batch 1, k = 4096; layer 0 all-retrieval,
layers 1..35 with 3 retrieval heads) with every input already resident in HBM, run the way a
model has to run it: LAYER AFTER LAYER, layer l's output complete before layer l+1 starts
(Alg. 1 computes the next layer's query from it).  That is lychee_decode_step in
LYCHEE_STEP_LAYERWISE mode: one launch per layer.  Prints ONE JSON line.

  value         microseconds per step (whole job, one GPU)
  roofline      the layer launch (lychee_layer_kernel, all of the step's bytes): algorithmic bytes
                per launch / its average duration, measured with HIP events on the launch
                stream, against the 8 TB/s HBM peak
  cpu_baseline  the fp64 CPU oracle timed on one whole step of the same workload
  phased_*      the same step when all 36 queries are known before it starts (not what a model
                can call): five pooled launches, and the roofline of its streaming launch

--secondary prints one JSON line per secondary configuration (c1, c2, c4, the c5 sweep, the
kernel-study grid, the selection rules): cold (KV copies rotated past the 256 MB cache) and warm,
median and minimum of >= 50 iterations, against the dense call on the same buffers; then the model
loop (deferred layer calls back to back) over context lengths from 8K to 128K.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "lychee_layer_kernel_c3_pmc.txt")
CSRC = os.path.join(ROOT, "paper_2602_04541_amd", "csrc")


def source_stamp() -> str:
    """A short hash of the kernel sources: a counter summary is only quoted for the build it was taken on."""
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            h.update(open(os.path.join(CSRC, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic():
    """HBM bytes per layer launch from the committed rocprofv3 --pmc summary, if it was taken on these sources."""
    try:
        fields = {}
        for line in open(TRAFFIC_FILE):
            if ":" in line:
                key, val = line.split(":", 1)
                fields[key.strip()] = val.strip()
        if fields.get("source_stamp") != source_stamp():
            return None
        return int(float(fields["traffic_bytes_per_launch"]))
    except (OSError, KeyError, ValueError):
        return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debug)")
    ap.add_argument("--k", type=int, default=0, help="override the budget (the c5 sweep)")
    ap.add_argument("--retrieval", type=int, default=0, help="override the retrieval heads per layer (the c5 sweep)")
    ap.add_argument("--ks", default="", metavar="BATCH,CONTEXT,SPARSE_GROUPS",
                    help="the kernel-study shape of Sec. 4.3.2 instead of a named workload "
                         "(one layer, block size 64, 90 %% block sparsity), e.g. 8,131072,8")
    ap.add_argument("--block", action="store_true",
                    help="block-granular sets (App. C): the budget becomes k/64 blocks of 64 positions")
    ap.add_argument("--wg-per-cu", type=int, default=0)
    ap.add_argument("--tail", type=int, default=-1)
    ap.add_argument("--gather-block", type=int, default=0)
    ap.add_argument("--phased", action="store_true", help="time the phased step (all queries known in advance) as `value`")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="skip the dense legs, the other step order and the layer calls")
    ap.add_argument("--secondary", action="store_true", help="the secondary configurations, one JSON line each")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not served (the path has no "
              "multi-GPU leg)" % args.gpus, file=sys.stderr)
        return 2
    if args.secondary:
        return secondary(args)

    import numpy as np
    import torch
    from paper_2602_04541_amd import binding as lb
    from paper_2602_04541_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    if args.ks:
        ks_batch, ks_ctx, ks_sparse = (int(x) for x in args.ks.split(","))
        w = wl.kernel_study(ks_batch, ks_ctx, ks_sparse)
        args.block = True
    else:
        w = wl.WORKLOADS[args.workload]
    if args.k:
        w = wl.scaled(w, k=args.k)
    if args.retrieval:
        w = wl.scaled(w, n_retrieval=args.retrieval)
    n_layers = args.layers or w.n_layers
    ctx = lb.Context(0)
    if args.wg_per_cu:
        ctx.set_option(lb.OPT_WG_PER_CU, args.wg_per_cu)
    if args.tail >= 0:
        ctx.set_option(lb.OPT_TAIL_PERMILLE, args.tail)
    if args.gather_block:
        ctx.set_option(lb.OPT_GATHER_BLOCK, args.gather_block)

    t_gen = time.perf_counter()
    layers = [wl.make_layer(w, layer=l, device=dev) for l in range(n_layers)]
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    masks = np.stack([ly.mask for ly in layers])
    lens_h = layers[0].lengths
    lens = torch.from_numpy(lens_h).to(dev)
    unit = 64 if args.block else 1          # positions one set entry names
    k_set = w.k if args.ks else max(1, w.k // unit)   # entries per set (the study's k counts blocks)
    shape = lb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.max_len, k_set, kv=layers[0].k_cache,
                          block_size=unit)
    ws = lb.alloc_workspace(shape, dev, n_layers=n_layers)
    outs = [torch.zeros_like(ly.q) for ly in layers]
    idx_final = torch.zeros((w.batch, w.n_kv_heads, k_set), dtype=torch.int32, device=dev)
    idx0 = None
    if not masks[0].all():      # single-layer workloads: some inherited sets to gather from
        idx0_h = np.tile(np.arange(k_set, dtype=np.int32), (w.batch, w.n_kv_heads, 1))
        for b in range(w.batch):
            idx0_h[b] = np.minimum(idx0_h[b], (int(lens_h[b]) - 1) // unit)
        if args.ks:             # a seeded tenth of the blocks per (sequence, KV head), ascending
            rng = np.random.Generator(np.random.Philox(key=wl.BASE_SEED + 6))
            n_units = (w.max_len + unit - 1) // unit
            for b in range(w.batch):
                for g in range(w.n_kv_heads):
                    idx0_h[b, g] = np.sort(rng.choice(n_units, size=k_set, replace=False))
        idx0 = torch.from_numpy(idx0_h).to(dev)
    qs = [ly.q for ly in layers]
    ks = [ly.k_cache for ly in layers]
    vs = [ly.v_cache for ly in layers]

    def hybrid_step():
        ctx.decode_step(shape, qs, ks, vs, masks, idx0, outs, idx_final, lens, ws)

    def dense_step():
        ctx.dense_decode_step(shape, qs, ks, vs, outs, lens, ws)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def set_mode(phased):
        ctx.set_option(lb.OPT_STEP_MODE, lb.STEP_PHASED if phased else lb.STEP_LAYERWISE)

    def launch_times(fn, steps):
        """Per-launch durations by launch class, HIP events on the launch stream."""
        ctx.timing_enable(True)
        for _ in range(steps):
            fn()
        ms, n = ctx.timing_read()
        ctx.timing_enable(False)
        return ms, n

    names = ["stream", "gather", "threshold", "select", "combine"]
    # ---- the timed region: exactly `steps` hybrid decode steps -------------------------
    set_mode(args.phased)
    sec = timed(hybrid_step, args.steps, args.warmup)
    ms_cls, n_cls = launch_times(hybrid_step, args.steps)
    stream_us = 1e3 * ms_cls[lb.KERNEL_STREAM] / max(1, n_cls[lb.KERNEL_STREAM])
    launches_per_step = {name: n_cls[i] // args.steps for i, name in enumerate(names)}

    # ---- the other step order, the dense kernel in both orders ----------------------------
    other_sec = dense_sec = dense_other_sec = None
    other_ms = other_n = None
    if not args.quick:
        set_mode(not args.phased)
        other_sec = timed(hybrid_step, max(3, args.steps // 3), 5)
        other_ms, other_n = launch_times(hybrid_step, max(3, args.steps // 3))
        dense_other_sec = timed(dense_step, max(3, args.steps // 3), 3)
        set_mode(args.phased)
        dense_sec = timed(dense_step, max(3, args.steps // 3), 3)
    # ---- the same layers through per-layer calls, as a model makes them: calls that leave their
    #      select pending (one launch each), and plain calls (their select is a launch of its own) ----
    calls_sec = deferred_sec = None
    if not args.quick and n_layers > 1 and masks[0].all():
        ws2 = lb.alloc_workspace(shape, dev, n_layers=2)
        pair = [torch.zeros_like(idx_final) for _ in range(2)]

        def layer_calls(deferred):
            call = ctx.decode_attn_deferred if deferred else ctx.decode_attn
            for l in range(n_layers):
                call(shape, qs[l], ks[l], vs[l], masks[l], pair[(l - 1) % 2] if l else None, outs[l],
                     pair[l % 2], lens, ws2)
            if deferred:
                ctx.select_flush()
        calls_sec = timed(lambda: layer_calls(False), max(3, args.steps // 3), 2)
        deferred_sec = timed(lambda: layer_calls(True), max(3, args.steps // 3), 2)
        del ws2
    # ---- a streaming-read ceiling: ONE launch of a plain read kernel over 2 GiB ---------------
    probe_bytes = 2 << 30
    probe_src = torch.empty(probe_bytes, dtype=torch.uint8, device=dev)
    probe_src.random_(0, 255)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    probe_us = []
    for it in range(6):
        ev[0].record()
        ctx.probe_read(probe_src, probe_bytes, sink)
        ev[1].record()
        torch.cuda.synchronize()
        if it:
            probe_us.append(ev[0].elapsed_time(ev[1]) * 1e3)
    read_ceiling = probe_bytes / (min(probe_us) * 1e-6) / 1e9
    # one plain copy of known size (reads and writes 256 MiB): the yardstick that the
    # FETCH_SIZE / WRITE_SIZE counters of a profiler run are scaled by
    ctx.probe_copy(probe_src[256 << 20:], probe_src, 256 << 20)
    torch.cuda.synchronize()
    del probe_src

    # ---- algorithmic bytes ---------------------------------------------------------------
    # per step: every K+V row streamed or gathered (512 B), the index sets, q and out.  Not
    # counted, although the library moves them: the threshold sample's K rows (256 B each,
    # 2048 per score row) and the candidate lists (8 B per candidate, written and read once)
    w_rows = wl.scaled(w, k=w.k * 64) if args.ks else w   # the budget in cache rows, for the byte counts
    step_bytes = sum(wl.algorithmic_bytes(w_rows, masks[l], lens_h) for l in range(n_layers))
    dense_bytes = n_layers * wl.dense_bytes(w, lens_h)
    G = w.group
    rows_streamed = 0
    rows_gathered = 0
    for l in range(n_layers):
        n_r = sum(1 for g in range(w.n_kv_heads) if masks[l][g * G:(g + 1) * G].any())
        n_s = sum(1 for g in range(w.n_kv_heads) if (masks[l][g * G:(g + 1) * G] == 0).any())
        rows_streamed += sum(n_r * int(L) for L in lens_h)
        rows_gathered += sum(n_s * min(w_rows.k, int(L)) for L in lens_h)
    qo_bytes = n_layers * w.batch * w.n_q_heads * 256
    n_stream_launches = max(1, launches_per_step["stream"])
    if args.phased:     # the streaming launch of the phased step: every layer's streamed rows, and q
        kernel_bytes = rows_streamed * 512 + qo_bytes
        kernel_name = "lychee_pool_kernel<true, false, true> (the streaming launch of the phased step)"
    else:               # the layer launches: a layer's streamed and gathered rows, q
        kernel_bytes = (rows_streamed + rows_gathered) * 512 + qo_bytes
        kernel_name = "lychee_layer_kernel<true, 1> (one launch per layer: thresholds, streaming, gathers, " \
                      "combine, the previous layer's select)"
    kernel_bytes /= n_stream_launches
    achieved = kernel_bytes / (stream_us * 1e-6) / 1e9 if stream_us > 0 else 0.0
    default_run = args.workload == "c3" and not (args.phased or args.layers or args.k or args.retrieval
                                                 or args.block or args.ks)
    traffic = measured_traffic() if default_run else None

    result = {
        "metric": "us per decode-step attention (all layers) at 128K",
        "value": round(sec * 1e6, 2),
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: %d layers, B%d, %dq/%dkv heads, d128, context %d, k %d, %s" % (
                                   w.name, n_layers, w.batch, w.n_q_heads, w.n_kv_heads, w.max_len, w.k,
                                   "layer 0 all-retrieval then %d retrieval heads per layer" % w.n_retrieval
                                   if w.first_layer_all_retrieval else
                                   "%d retrieval heads" % int(masks[0].sum())),
                   "step_mode": "phased (all queries given before the step)" if args.phased else
                                "layer after layer (a layer's output complete before the next layer starts)",
                   "sets": "blocks of 64 positions" if args.block else "positions"},
        "step_algorithmic_bytes": step_bytes,
        "step_achieved_gbps": round(step_bytes / sec / 1e9, 1),
        "step_hbm_frac": round(step_bytes / sec / 1e9 / HBM_PEAK_GBPS, 4),
        "read_ceiling_gbps": round(read_ceiling, 1),
        "launches_per_step": launches_per_step,
        "launch_us_per_step": {name: round(1e3 * ms_cls[i] / args.steps, 2) for i, name in enumerate(names)},
        "paper_context": "paper reports up to 2.7x end-to-end TPOT speed-up over full attention at "
                         "128K, batch 1, budget 4096 (Sec. 4.3.1; GPU of that run not stated, kernel "
                         "study on one NVIDIA A800)",
        "roofline": {"bound": "hbm", "kernel": kernel_name,
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_note": None if traffic is not None or not default_run else
                                     "no counter summary for this build under profiles/ (source stamp %s)" % source_stamp(),
                     "avg_launch_us": round(stream_us, 2),
                     "launches_per_step": n_stream_launches,
                     "algorithmic_bytes_per_launch": int(kernel_bytes),
                     "frac_of_read_ceiling": round(achieved / read_ceiling, 4) if read_ceiling > 0 else None},
        "gen_seconds": round(t_gen, 1),
        # score rows that the select had to rank from all of their scores (threshold too high,
        # candidate list full) in everything this process ran: time lost, not correctness
        "select_fallbacks": list(ctx.select_stats()),
    }
    if other_sec is not None:
        # the other step order, and the dense kernel on identical buffers in both orders
        mine, other = ("phased", "layerwise") if args.phased else ("layerwise", "phased")
        result["%s_us" % other] = round(other_sec * 1e6, 2)
        result["%s_hbm_frac" % other] = round(step_bytes / other_sec / 1e9 / HBM_PEAK_GBPS, 4)
        n_o = max(1, other_n[lb.KERNEL_STREAM])
        o_us = 1e3 * other_ms[lb.KERNEL_STREAM] / n_o
        o_bytes = ((rows_streamed * 512 + qo_bytes) if not args.phased else
                   ((rows_streamed + rows_gathered) * 512 + qo_bytes)) / (n_o / max(3, args.steps // 3))
        result["%s_stream_launch" % other] = {"avg_launch_us": round(o_us, 2),
                                              "algorithmic_bytes_per_launch": int(o_bytes),
                                              "frac": round(o_bytes / (o_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
        result["dense_%s_us" % mine] = round(dense_sec * 1e6, 2)
        result["dense_%s_us" % other] = round(dense_other_sec * 1e6, 2)
        result["dense_achieved_gbps"] = round(dense_bytes / dense_sec / 1e9, 1)
        result["speedup_vs_dense_%s" % mine] = round(dense_sec / sec, 3)
        result["speedup_vs_dense_%s" % other] = round(dense_other_sec / other_sec, 3)
    if calls_sec is not None:
        # the step as n_layers lychee_decode_attn_deferred calls + a flush, and as lychee_decode_attn calls
        result["layer_calls_deferred_select_us"] = round(deferred_sec * 1e6, 2)
        result["layer_calls_us"] = round(calls_sec * 1e6, 2)

    # ---- the CPU oracle on a bounded sample of the same workload --------------------------
    if not args.no_cpu_baseline:
        from oracle import lychee_oracle as lo
        # every layer of the step, chained through its sets exactly like the GPU step; the
        # device-to-host copies of the cache are outside the timed regions
        t_cpu = 0.0
        idx = None if masks[0].all() else idx0.cpu().numpy()
        for l in range(n_layers):
            ly = layers[l]
            qb, kb, vb = (wl.bf16_bits(t) for t in (ly.q, ly.k_cache, ly.v_cache))
            t0 = time.perf_counter()
            _, idx, _ = lo.decode_attn(qb, kb, vb, masks[l], k_set, idx, lens_h, block=unit)
            t_cpu += time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(t_cpu * 1e6, 0), "unit": "us", "cores": lo.num_threads(),
                                  "kind": "oracle",
                                  "sample": "one whole step: all %d layers of the same workload, sets "
                                            "chained layer to layer (%.2f s of oracle time)" % (n_layers, t_cpu)}
    print(json.dumps(result), flush=True)
    ctx.close()
    return 0


def secondary(args) -> int:
    """The secondary configurations: single layer calls (lychee_decode_attn_deferred + lychee_select_flush,
    i.e. the layer launch and the select launch), cold and warm, against the dense call."""
    import numpy as np
    import torch
    from paper_2602_04541_amd import binding as lb
    from paper_2602_04541_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    ctx = lb.Context(0)
    iters = max(50, args.steps)
    cases = [("c1", wl.WORKLOADS["c1"], {}), ("c2", wl.WORKLOADS["c2"], {}), ("c4", wl.WORKLOADS["c4"], {})]
    for n_r in (1, 4, 32):
        for k in (64, 1024, 4096, 8192, 131072):
            if n_r == 32 and k != 4096:
                continue
            cases.append(("c5 r%d k%d" % (n_r, k), wl.scaled(wl.WORKLOADS["c5"], k=k, n_retrieval=n_r), {}))
    for batch, context in ((1, 16384), (1, 131072), (8, 16384), (8, 131072)):
        for sparse in (4, 6, 8):
            cases.append(("ks b%d L%d s%d/8" % (batch, context, sparse), wl.kernel_study(batch, context, sparse),
                          {"block_size": 64}))
    c5 = wl.WORKLOADS["c5"]
    cases.append(("c5 ratio keep 3%", c5, {"keep_ppm": 30000}))
    cases.append(("c5 threshold 1e-4", c5, {"prob_rule": lb.RULE_THRESHOLD, "prob_param": 1e-4}))
    cases.append(("c5 top-p 0.9", c5, {"prob_rule": lb.RULE_TOP_P, "prob_param": 0.9}))

    for name, w, kw in cases:
        unit = kw.get("block_size", 1) or 1
        probe = wl.make_layer(w, layer=0, device=dev)
        kv_bytes = 2 * probe.k_cache.numel() * 2
        # cold: rotate through copies of the cache that together exceed the 256 MB cache several times
        n_copies = int(min(400, max(1, -(-(3 << 29) // kv_bytes))))
        copies = [probe] + [wl.make_layer(w, layer=1 + i, device=dev) for i in range(n_copies - 1)]
        mask = probe.mask
        lens_h = probe.lengths
        lens = torch.from_numpy(lens_h).to(dev)
        shape = lb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.max_len, w.k, kv=probe.k_cache, **kw)
        ws = lb.alloc_workspace(shape, dev, n_layers=2)
        out = torch.zeros_like(probe.q)
        idx_out = torch.zeros((w.batch, w.n_kv_heads, w.k), dtype=torch.int32, device=dev)
        idx_in = None
        if not mask.all():
            n_units = [max(1, -(-int(L) // unit)) for L in lens_h]
            rng = np.random.Generator(np.random.Philox(key=wl.BASE_SEED + 6))
            idx_h = np.full((w.batch, w.n_kv_heads, w.k), -1, np.int32)
            for b in range(w.batch):
                n = min(w.k, n_units[b])
                for g in range(w.n_kv_heads):
                    idx_h[b, g, :n] = np.sort(rng.choice(n_units[b], size=n, replace=False))
            idx_in = torch.from_numpy(idx_h).to(dev)

        def hybrid(ly):
            ctx.decode_attn_deferred(shape, ly.q, ly.k_cache, ly.v_cache, mask, idx_in, out, idx_out, lens, ws)
            ctx.select_flush()

        def dense(ly):
            ctx.dense_decode_attn(shape, ly.q, ly.k_cache, ly.v_cache, out, lens, ws)

        def sample(fn, rotate):
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
            for i in range(10):
                fn(copies[i % n_copies] if rotate else copies[0])
            for i in range(iters):
                ev[i][0].record()
                fn(copies[i % n_copies] if rotate else copies[0])
                ev[i][1].record()
            torch.cuda.synchronize()
            t = np.array([a.elapsed_time(b) * 1e3 for a, b in ev])
            return float(np.median(t)), float(t.min())

        w_rows = wl.scaled(w, k=w.k * unit)
        bytes_h = wl.algorithmic_bytes(w_rows, mask, lens_h)
        bytes_d = wl.dense_bytes(w, lens_h)
        cold = sample(hybrid, True)
        warm = sample(hybrid, False)
        dcold = sample(dense, True)
        dwarm = sample(dense, False)
        print(json.dumps({
            "config": name, "shape": "B%d %dq/%dkv L%d k%d%s, %d retrieval heads" % (
                w.batch, w.n_q_heads, w.n_kv_heads, w.max_len, w.k, " blocks" if unit == 64 else "", int(mask.sum())),
            "iters": iters, "kv_copies_rotated": n_copies,
            "hybrid_cold_us_median_min": [round(x, 1) for x in cold], "hybrid_warm_us_median_min": [round(x, 1) for x in warm],
            "dense_cold_us_median_min": [round(x, 1) for x in dcold], "dense_warm_us_median_min": [round(x, 1) for x in dwarm],
            "algorithmic_bytes": int(bytes_h), "dense_bytes": int(bytes_d),
            "hybrid_cold_gbps": round(bytes_h / cold[0] / 1e3, 1), "hybrid_cold_hbm_frac": round(bytes_h / cold[0] / 1e3 / HBM_PEAK_GBPS, 4),
            "dense_cold_gbps": round(bytes_d / dcold[0] / 1e3, 1),
            "speedup_vs_dense_cold": round(dcold[0] / cold[0], 3)}), flush=True)
        del copies, probe, ws
        torch.cuda.empty_cache()
    # The model loop over context lengths: deferred layer calls back to back (each call's select inside the next
    # call's launch), 8 layers of the c3 head layout (3 retrieval heads per layer), rotating through the layers'
    # caches; against the dense call on the same caches.  Microseconds per layer, whole loop / layers.
    c3 = wl.WORKLOADS["c3"]
    for context in (8192, 16384, 32768, 65536, 131072):
        for k in (1024, 4096):
            if 2 * k > context:
                continue
            w = wl.scaled(c3, max_len=context, k=k, n_layers=9)
            layers = [wl.make_layer(w, layer=l, device=dev, l_cap=context) for l in range(1, 9)]
            lens = torch.from_numpy(layers[0].lengths).to(dev)
            shape = lb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, context, k, kv=layers[0].k_cache)
            ws = lb.alloc_workspace(shape, dev, n_layers=2)
            out = torch.zeros_like(layers[0].q)
            pair = [torch.zeros((w.batch, w.n_kv_heads, k), dtype=torch.int32, device=dev) for _ in range(2)]
            for t in pair:
                t[:] = torch.arange(k, dtype=torch.int32, device=dev) * (context // k)

            def loop_hybrid():
                for l, ly in enumerate(layers):
                    ctx.decode_attn_deferred(shape, ly.q, ly.k_cache, ly.v_cache, ly.mask, pair[l & 1], out, pair[(l + 1) & 1], lens, ws)

            def loop_dense():
                for ly in layers:
                    ctx.dense_decode_attn(shape, ly.q, ly.k_cache, ly.v_cache, out, lens, ws)

            def per_layer(fn):
                t = []
                for rep in range(3 + 10):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(4):
                        fn()
                    e1.record()
                    torch.cuda.synchronize()
                    if rep >= 3:
                        t.append(e0.elapsed_time(e1) * 1e3 / (4 * len(layers)))
                return round(float(np.median(t)), 1), round(float(min(t)), 1)

            hyb = per_layer(loop_hybrid)
            ctx.select_flush()
            den = per_layer(loop_dense)
            mask_bytes = np.mean([wl.algorithmic_bytes(w, ly.mask, ly.lengths) for ly in layers])
            print(json.dumps({
                "config": "model loop L%d k%d" % (context, k),
                "shape": "B1 32q/8kv, 8 layers with 3 retrieval heads each, deferred calls back to back",
                "hybrid_us_per_layer_median_min": list(hyb), "dense_us_per_layer_median_min": list(den),
                "algorithmic_bytes_per_layer": int(mask_bytes),
                "hybrid_hbm_frac": round(mask_bytes / hyb[0] / 1e3 / HBM_PEAK_GBPS, 4),
                "speedup_vs_dense": round(den[0] / hyb[0], 3)}), flush=True)
            del layers, ws
            torch.cuda.empty_cache()
    print(json.dumps({"select_fallbacks": list(ctx.select_stats()), "wait_timeouts": ctx.wait_timeouts()}), flush=True)
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
