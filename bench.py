#!/usr/bin/env python3
"""Benchmark of the decode-step hybrid-head attention on one MI355X.

A *step* is the attention of one whole decode step on the Qwen3-8B-shaped 128K workload
(36 layers, 32 query / 8 KV heads, head dim 128, batch 1, k = 4096; layer 0 all-retrieval,
layers 1..35 with 3 retrieval heads): one call of lychee_decode_step with every input
already resident in HBM.  Prints ONE JSON line.

  value      microseconds per step (whole job, one GPU)
  roofline   the streaming launch of the work-unit kernel (it moves > 90 % of the bytes):
             algorithmic bytes of that launch / its duration measured with HIP events on the
             launch stream, against the 8 TB/s HBM peak
  cpu_baseline  the fp64 CPU oracle timed on one whole step of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "lychee_pool_kernel_c3_stream_pmc.txt")


def measured_traffic():
    """HBM bytes per streaming launch from the committed rocprofv3 --pmc summary, if any."""
    try:
        for line in open(TRAFFIC_FILE):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1]))
    except OSError:
        pass
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
    ap.add_argument("--layerwise", action="store_true", help="time the layer-after-layer step as `value`")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="skip the dense and layerwise legs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not served (the path has no "
              "multi-GPU leg)" % args.gpus, file=sys.stderr)
        return 2

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

    def set_mode(layerwise):
        ctx.set_option(lb.OPT_STEP_MODE, lb.STEP_LAYERWISE if layerwise else lb.STEP_PHASED)

    # ---- the timed region: exactly `steps` hybrid decode steps -------------------------
    set_mode(args.layerwise)
    sec = timed(hybrid_step, args.steps, args.warmup)

    # ---- per-launch durations with HIP events on the launch stream (same steps again) ---
    ctx.timing_enable(True)
    for _ in range(args.steps):
        hybrid_step()
    ms_cls, n_cls = ctx.timing_read()
    ctx.timing_enable(False)
    stream_us = 1e3 * ms_cls[lb.KERNEL_STREAM] / max(1, n_cls[lb.KERNEL_STREAM])
    launches_per_step = {name: n_cls[i] // args.steps for i, name in
                         enumerate(["stream", "gather", "threshold", "select", "combine"])}

    # ---- the other step order, the dense kernel, the streaming-read ceiling ---------------
    other_sec = dense_sec = dense_other_sec = None
    if not args.quick:
        set_mode(not args.layerwise)
        other_sec = timed(hybrid_step, max(3, args.steps // 3), 1)
        dense_other_sec = timed(dense_step, max(3, args.steps // 3), 1)
        set_mode(args.layerwise)
        dense_sec = timed(dense_step, max(3, args.steps // 3), 1)
    # ---- the same layers through per-layer calls, as a model that computes q[l+1] from
    #      out[l] has to make them: plain calls, and calls that leave their select pending -----
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
        calls_sec = timed(lambda: layer_calls(False), max(3, args.steps // 3), 1)
        deferred_sec = timed(lambda: layer_calls(True), max(3, args.steps // 3), 1)
        del ws2
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_bytes = ks[0].numel() * 2
    n_probe = min(n_layers, 8)

    def probe():
        for l in range(n_probe):
            ctx.probe_read(ks[l], probe_bytes, sink)
    probe_sec = timed(probe, 5, 1)
    read_ceiling = probe_bytes * n_probe / probe_sec / 1e9
    # one plain copy of known size (reads and writes probe_bytes): the yardstick that the
    # FETCH_SIZE / WRITE_SIZE counters of a profiler run are scaled by
    copy_dst = torch.empty_like(ks[0])
    ctx.probe_copy(copy_dst, ks[0], probe_bytes)
    torch.cuda.synchronize()
    del copy_dst

    # ---- algorithmic bytes ---------------------------------------------------------------
    # per step: every K+V row streamed or gathered (512 B), the index sets, q and out.  Not
    # counted, although the library moves them: the threshold sample's K rows (256 B each,
    # 2048 per score row) and the candidate lists (8 B per candidate, written and read once)
    w_rows = wl.scaled(w, k=w.k * 64) if args.ks else w   # the budget in cache rows, for the byte counts
    step_bytes = sum(wl.algorithmic_bytes(w_rows, masks[l], lens_h) for l in range(n_layers))
    dense_bytes = n_layers * wl.dense_bytes(w, lens_h)
    # per streaming launch: 512 B of K+V per streamed row, plus q
    G = w.group
    rows_streamed = 0
    rows_gathered = 0
    for l in range(n_layers):
        n_r = sum(1 for g in range(w.n_kv_heads) if masks[l][g * G:(g + 1) * G].any())
        n_s = sum(1 for g in range(w.n_kv_heads) if (masks[l][g * G:(g + 1) * G] == 0).any())
        rows_streamed += sum(n_r * int(L) for L in lens_h)
        rows_gathered += sum(n_s * min(w_rows.k, int(L)) for L in lens_h)
    n_stream_launches = max(1, launches_per_step["stream"])
    if args.layerwise:          # the streaming launch of a layer also carries its gathers
        stream_bytes = (rows_streamed + rows_gathered) * 512
    else:
        stream_bytes = rows_streamed * 512
    stream_bytes = (stream_bytes + n_layers * w.batch * w.n_q_heads * 256) / n_stream_launches
    achieved = stream_bytes / (stream_us * 1e-6) / 1e9 if stream_us > 0 else 0.0
    default_run = args.workload == "c3" and not (args.layerwise or args.layers or args.k or args.retrieval
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
                   "step_mode": "layerwise" if args.layerwise else "phased",
                   "sets": "blocks of 64 positions" if args.block else "positions"},
        "step_algorithmic_bytes": step_bytes,
        "step_achieved_gbps": round(step_bytes / sec / 1e9, 1),
        "step_hbm_frac": round(step_bytes / sec / 1e9 / HBM_PEAK_GBPS, 4),
        "read_ceiling_gbps": round(read_ceiling, 1),
        "launches_per_step": launches_per_step,
        "launch_us_per_step": {name: round(1e3 * ms_cls[i] / args.steps, 2) for i, name in
                               enumerate(["stream", "gather", "threshold", "select", "combine"])},
        "paper_context": "paper reports up to 2.7x end-to-end TPOT speed-up over full attention at "
                         "128K, batch 1, budget 4096 (Sec. 4.3.1; GPU of that run not stated, kernel "
                         "study on one NVIDIA A800)",
        "roofline": {"bound": "hbm", "kernel": "lychee_pool_kernel<true, false, true> (the streaming launch of the phased step)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "avg_launch_us": round(stream_us, 2),
                     "algorithmic_bytes_per_launch": int(stream_bytes)},
        "gen_seconds": round(t_gen, 1),
        # score rows that the select had to rank from all of their scores (threshold too high,
        # candidate list full) in everything this process ran: time lost, not correctness
        "select_fallbacks": list(ctx.select_stats()),
    }
    if other_sec is not None:
        # the dense kernel on identical buffers, in the same step order as `value` and in the other
        other = "layerwise" if not args.layerwise else "phased"
        result["%s_us" % other] = round(other_sec * 1e6, 2)
        result["dense_us"] = round(dense_sec * 1e6, 2)
        result["dense_%s_us" % other] = round(dense_other_sec * 1e6, 2)
        result["dense_achieved_gbps"] = round(dense_bytes / dense_sec / 1e9, 1)
        result["speedup_vs_dense"] = round(dense_sec / sec, 3)
        result["speedup_vs_dense_%s" % other] = round(dense_other_sec / other_sec, 3)
    if calls_sec is not None:
        # the step as n_layers lychee_decode_attn calls, and as lychee_decode_attn_deferred calls + a flush
        result["layer_calls_us"] = round(calls_sec * 1e6, 2)
        result["layer_calls_deferred_select_us"] = round(deferred_sec * 1e6, 2)

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


if __name__ == "__main__":
    sys.exit(main())
