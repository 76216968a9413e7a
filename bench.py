#!/usr/bin/env python3
"""Benchmark of the Ada-KV per-layer compression step on one MI355X.

One step = one pass of the whole hot path (adakv_score + adakv_allocate + adakv_select +
adakv_compact, one stream, no host synchronisation in between) over one seeded synthetic
layer.  Inputs are resident in HBM before the timed region; the step rotates over several
distinct input sets (more than a gigabyte in total, against 256 MB of memory-side cache) so
that the K stream really comes from HBM.

`--path decode` measures the decode side of the flattened cache instead (one step = one
adakv_decode_step, i.e. append + decode attention, over the layer's compressed cache, built by the same
compression with `--budget-frac` of every prefix kept); the default is the compression step.

Prints ONE JSON line.  `value` is prefix tokens compressed per second (the layer's n divided
by the time of a step).  `roofline` describes the dominant kernel, timed live with a pair of
events attached to its launch on the launch stream (adakv_trace_arm; they receive the kernel's
own start and end time) in a second pass over the same inputs; `cpu_baseline` is the fp64 CPU
oracle on the same layer.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published peak
MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 / fp16 MFMA, published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0
PROFILES = os.path.join(ROOT, "profiles")


def measured_traffic(summary):
    """HBM bytes per launch (fetched + written) of every kernel listed in a rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE summary under profiles/ (written from the counter CSVs, both counters
    scaled by what they read for a 1 GiB copy): {name as bench.py traces it: bytes}, or {} when
    the summary is not there.  Rows: | `kernel` | bench.py name | launches | FETCH KiB | fetched MiB
    | WRITE KiB | written MiB | avg us |."""
    path = os.path.join(PROFILES, summary)
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 8 and cells[0].startswith("`"):
            try:
                out[cells[1]] = int((float(cells[4]) + float(cells[6])) * 2 ** 20)
            except ValueError:
                pass
    return out


def median_step_ms(torch, step, n_steps):
    """Median over n_steps of the time of one step, from a pair of events around each on the
    stream the step is issued on."""
    pairs = []
    for i in range(n_steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        step(i)
        e1.record()
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in pairs)
    return ts[len(ts) // 2]


def algorithmic_bytes(wl, kept_rows):
    """Bytes the path has to move per layer call, per stage (one read of K for scoring, one
    write and two reads of the scores, one read and one write of every kept K and V row)."""
    esz = 4 if str(wl.dtype).endswith("float32") else 2
    n_tot = wl.total_prefix_tokens
    k_stream = n_tot * wl.h_kv * wl.d * esz
    sc = n_tot * wl.h_kv * 4
    gather = kept_rows * wl.d * esz * 2 * 2
    return {"score": k_stream + sc, "allocate": sc, "select": sc + kept_rows * 4,
            "compact": gather + kept_rows * 4, "k_stream": k_stream}


def traced_pass(adakv, torch, step, n_steps, kernels_per_step):
    """Per-kernel durations from event pairs attached to the launches.  Steps run back to back
    inside one trace (as many as its 256 events hold) with one synchronisation per batch, so the
    kernels are timed in the same stream of work as in the throughput measurement."""
    per_kernel, order = {}, []
    batch = max(1, 256 // (2 * kernels_per_step))
    done = 0
    while done < n_steps:
        todo = min(batch, n_steps - done)
        with adakv.KernelTrace(256) as tr:
            for i in range(done, done + todo):
                step(i)
        torch.cuda.synchronize()
        for name, us in tr.durations_us():
            if name not in per_kernel:
                per_kernel[name] = []
                order.append(name)
            per_kernel[name].append(us)
        done += todo
    return per_kernel, order


def calibrate_copy(torch, dev):
    """Three 1 GiB device-to-device copies: a known number of bytes for scaling rocprofv3's
    FETCH_SIZE / WRITE_SIZE counters."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def bench_decode(args):
    """One step = adakv_decode_step (append + attention) for every sequence and head of one
    layer, on the cache the compression step produced."""
    import numpy as np
    import torch

    import paper_2407_11550_amd as adakv
    from paper_2407_11550_amd import synth

    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = synth.workload(args.workload, alpha=args.alpha)
    if args.budget_frac is not None:
        wl.B = [wl.h_kv * (wl.w + max(1, int(round(args.budget_frac * nb)))) for nb in wl.n]
    layer = adakv.Layer.from_workload(wl)
    trace_steps = min(args.steps, 50)
    hr = args.warmup + args.steps + trace_steps
    sets = []
    for i in range(args.sets):
        q, K, V = synth.generate(wl, layer=i, device=dev)
        res = adakv.compress(layer, q, K, V)
        Kc, Vc, seg_len = adakv.cache_build(layer, K, V, res["indices"], res["cu_seqlens"], hr)
        sets.append((Kc, Vc, res["cu_seqlens"], seg_len))
        del q, K, V, res
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    nsteps = 16
    qn, kn, vn = synth.decode_inputs(wl, nsteps, device=dev)
    ws = torch.empty(adakv.decode_workspace_bytes(layer, hr), dtype=torch.uint8, device=dev)
    out = torch.empty((wl.batch, wl.h_q, wl.d), dtype=torch.float32, device=dev)
    overflow = torch.zeros(1, dtype=torch.int32, device=dev)
    if args.calibrate_copy:
        calibrate_copy(torch, dev)

    def step(i):
        Kc, Vc, cu, seg_len = sets[i % len(sets)]
        t = i % nsteps
        adakv.decode_step(layer, qn[t], kn[t], vn[t], cu, hr, Kc, Vc, seg_len, overflow=overflow,
                          out=out, ws=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = 1000.0 * (t1 - t0) / args.steps
    per_kernel, order = traced_pass(adakv, torch, step, trace_steps, kernels_per_step=2)
    assert int(overflow.item()) == 0, "head-room too small for the number of steps"
    kernels = {k: float(np.mean(v)) for k, v in per_kernel.items()}
    esz = 4 if str(wl.dtype).endswith("float32") else 2
    rows = float(np.mean([int(s[3].sum().item()) for s in sets]))      # rows held at the end
    dom_bytes = rows * wl.d * esz * 2                                   # every K and V row once
    dom_us = max(kernels["decode_attn"], 1e-3)
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": "decode_attn", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(f"decode_{wl.name}_hbm_traffic.md").get("decode_attn")
                if args.budget_frac is None else None,
                "traffic_source": f"profiles/decode_{wl.name}_hbm_traffic.md",
                "algorithmic_bytes": int(dom_bytes), "avg_us": round(dom_us, 2)}
    cpu = None
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info

        from oracle import decode_oracle as D
        Kc, Vc, cu, seg_len = sets[0]
        Kd, Vd = Kc.double().cpu().numpy(), Vc.double().cpu().numpy()
        cuh, lens = cu.cpu().numpy(), seg_len.cpu().numpy()
        spent, done = 0.0, 0
        while spent < 10.0 and done < 64:
            qd = qn[done % nsteps].double().cpu().numpy()
            c0 = time.perf_counter()
            D.decode_attention(qd, Kd, Vd, cuh, hr, lens, wl.g)
            spent += time.perf_counter() - c0
            done += 1
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        cpu = {"value": round(done * float(lens.sum()) / spent, 1), "unit": "cached rows/s", "cores": threads,
               "kind": "oracle", "seconds": round(spent, 3),
               "sample": f"{done} decode attention step(s) over the whole cache of {wl.name} "
                         f"({int(lens.sum())} rows), fp64 numpy, the append not included"}
    print(json.dumps({
        "metric": "cached K/V rows attended/sec per layer (append + variable-length decode attention)",
        "value": round(rows / (ms_per_step * 1e-3), 1), "unit": "cached rows/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"torch.bfloat16": "bf16", "torch.float16": "f16"}.get(str(wl.dtype), "f32"), "data": "synthetic",
        "config": {"workload": wl.name + " (decode side)", "h_q": wl.h_q, "h_kv": wl.h_kv, "d": wl.d,
                   "n": wl.n, "w": wl.w, "B": wl.B, "alpha": wl.alpha, "batch": wl.batch,
                   "cached_rows": int(rows), "headroom": hr, "input_sets_rotated": len(sets)},
        "kernels_us": {k: round(kernels[k], 2) for k in order}, "roofline": roofline, "cpu_baseline": cpu}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama8b_128k",
                    help="llama8b_128k (the headline), llama8b_32k, llama8b_ragged, llama70b_128k, tiny")
    ap.add_argument("--alpha", type=float, default=None)
    ap.add_argument("--sets", type=int, default=5, help="distinct input sets rotated over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=1,
                    help="compress path: issue the layer calls round-robin on this many streams (each with "
                         "its own workspace and outputs), so that one layer's latency-bound selection kernels "
                         "run beside the next layer's sweeps; 1 (the default, the headline) = one layer at a time")
    ap.add_argument("--row-lse", action="store_true",
                    help="compress path: hand adakv_score the prefill attention's row log-sum-exp, "
                         "which removes the statistics sweep (not the headline configuration)")
    ap.add_argument("--pool-then-mean", action="store_true",
                    help="compress path: ADAKV_FLAG_POOL_THEN_MEAN, the printed order of Alg. 2 l.4 (pool every "
                         "window row, then average); not the headline configuration")
    ap.add_argument("--path", default="compress", choices=["compress", "decode"],
                    help="compress: the per-layer compression step (the headline); decode: append + "
                         "decode attention over the compressed cache")
    ap.add_argument("--budget-frac", type=float, default=None,
                    help="decode path: keep this fraction of every prefix instead of the workload's budget")
    ap.add_argument("--pyramid", type=float, default=None, metavar="RATIO",
                    help="compress path: treat the --sets input sets as consecutive layers and give them the "
                         "pyramidal variant's budgets (adakv_pyramid_budgets, first layer RATIO times the last, "
                         "mean = the workload's budget); not the headline configuration")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB device-to-device copy (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path has no multi-GPU part); "
                 "use --gpus 1")

    import numpy as np
    import torch

    import paper_2407_11550_amd as adakv
    from paper_2407_11550_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.path == "decode":
        return bench_decode(args)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = synth.workload(args.workload, alpha=args.alpha)
    flags = adakv.binding.ADAKV_FLAG_POOL_THEN_MEAN if args.pool_then_mean else 0
    layer = adakv.Layer.from_workload(wl, flags=flags)
    sets = [synth.generate(wl, layer=i, device=dev) for i in range(args.sets)]
    lses = [synth.prefill_row_lse(wl, q, K) if args.row_lse else None for q, K, _ in sets]
    # one layer description per input set: all alike, or the pyramidal variant's budgets per layer
    layers = [layer] * args.sets
    if args.pyramid is not None:
        wh = wl.w * wl.h_kv
        per_seq = [adakv.pyramid_budgets(args.sets, Bb - wh, args.pyramid) for Bb in wl.B]
        layers = []
        for l in range(args.sets):
            wll = synth.workload(args.workload, alpha=args.alpha)
            wll.B = [min(per_seq[b][l], wl.h_kv * wl.n[b]) + wh for b in range(wl.batch)]
            layers.append(adakv.Layer.from_workload(wll, flags=flags))
        layer = max(layers, key=lambda L: L.num_rows_out)          # sizes the output buffers
    def make_bufs():
        return (torch.empty(adakv.workspace_bytes(layer), dtype=torch.uint8, device=dev),
                dict(scores=torch.empty(layer.num_scores, dtype=torch.float32, device=dev),
                     budgets=torch.empty(layer.num_segments, dtype=torch.int32, device=dev),
                     cu_seqlens=torch.empty(layer.num_segments + 1, dtype=torch.int32, device=dev),
                     indices=torch.empty(layer.num_rows_out, dtype=torch.int32, device=dev),
                     K_out=torch.empty((layer.num_rows_out, wl.d), dtype=wl.dtype, device=dev),
                     V_out=torch.empty((layer.num_rows_out, wl.d), dtype=wl.dtype, device=dev)))

    # one workspace and one set of outputs per stream: calls that share them must be ordered
    lanes = [make_bufs() for _ in range(max(1, args.streams))]
    streams = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else [None]
    ws, bufs = lanes[0]

    if args.calibrate_copy:
        calibrate_copy(torch, dev)

    def step(i):
        q, K, V = sets[i % len(sets)]
        lane_ws, lane_bufs = lanes[i % len(lanes)]
        return adakv.compress(layers[i % len(sets)], q, K, V, row_lse=lses[i % len(sets)], ws=lane_ws,
                              bufs=lane_bufs, stream=streams[i % len(streams)])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = 1000.0 * (t1 - t0) / args.steps
    tokens = wl.total_prefix_tokens
    value = tokens / (ms_per_step * 1e-3)

    # ---- per-kernel durations, live, events on the launch stream (a second pass) ------------
    trace_steps = min(args.steps, 50)
    per_kernel, order = traced_pass(adakv, torch, step, trace_steps, kernels_per_step=16)
    kernels = {k: float(np.mean(v)) for k, v in per_kernel.items()}
    kept = int(np.mean([L.num_rows_out for L in layers]))
    alg = algorithmic_bytes(wl, kept)
    dominant = max(kernels, key=kernels.get)
    # bytes one launch of the dominant kernel has to move: a scoring sweep reads K once
    if dominant.startswith("score_") and dominant not in ("score_pool", "score_lse_combine"):
        dom_bytes = alg["k_stream"]
    elif dominant == "compact":
        dom_bytes = alg["compact"]
    else:
        dom_bytes = tokens * wl.h_kv * 4
    dom_us = max(kernels[dominant], 1e-3)
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    total_alg = alg["score"] + alg["allocate"] + alg["select"] + alg["compact"]
    flops = 2.0 * wl.g * wl.w * wl.d * wl.h_kv * tokens
    # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
    # counters read for a 1 GiB copy (profiles/llama8b_128k_hbm_traffic.md); only for the
    # workload and kernels that were profiled
    plain = (args.streams == 1 and not args.row_lse and args.pyramid is None and args.alpha is None
             and not args.pool_then_mean)
    per_kernel_traffic = measured_traffic(f"{wl.name}_hbm_traffic.md") if plain else {}
    traffic = per_kernel_traffic.get(dominant)
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": f"profiles/{wl.name}_hbm_traffic.md" if traffic else None,
                "algorithmic_bytes": dom_bytes, "avg_us": round(dom_us, 2)}
    # A scoring sweep does 2 g w d h flops per token on h d 2 bytes of K: g w flops per byte.  Past
    # the machine balance (dense 16-bit MFMA peak over HBM peak, 312 flops per byte) the sweep is
    # bound by the matrix cores and is priced against their peak; the HBM figure stays beside it.
    if (dominant in ("score_stats_mfma", "score_weights_mfma") and not str(wl.dtype).endswith("float32")
            and wl.g * wl.w > MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)):
        tflops = flops / (dom_us * 1e-6) / 1e12
        roofline = {"bound": "mfma", "kernel": dominant, "achieved": round(tflops, 1), "peak": MFMA_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(tflops / MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
                    "traffic_source": roofline["traffic_source"], "algorithmic_flops": flops,
                    "algorithmic_bytes": dom_bytes, "hbm_frac": roofline["frac"], "avg_us": round(dom_us, 2)}
    # counter traffic of the whole step (every kernel of it, from the same summary) over the bytes
    # the path has to move: what is above 1 is re-read or scratch traffic
    step_traffic = (sum(per_kernel_traffic[k] for k in order) if per_kernel_traffic
                    and all(k in per_kernel_traffic for k in order) else None)
    median_ms = median_step_ms(torch, step, max(50, min(args.steps, 200))) if args.streams == 1 else None

    # ---- what a kernel that only reads reaches here: the same K buffers, rotated the same way ---
    sink = torch.empty(adakv.PROBE_SINK_BYTES, dtype=torch.uint8, device=dev)
    for i in range(len(sets)):
        adakv.probe_read(sets[i][1], sink)
    with adakv.KernelTrace(128) as tr:
        for i in range(60):
            adakv.probe_read(sets[i % len(sets)][1], sink)
    torch.cuda.synchronize()
    probe_us = float(np.mean([us for _, us in tr.durations_us()]))
    probe_bytes = sets[0][1].numel() * sets[0][1].element_size()
    stream_read = {"kernel": "probe_read", "GB/s": round(probe_bytes / (probe_us * 1e-6) / 1e9, 1),
                   "bytes": probe_bytes, "avg_us": round(probe_us, 2),
                   "note": "plain 16-byte-per-lane read of the K buffers (window rows included), rotating "
                           "over the input sets like the step does"}
    if dominant.startswith("score_"):
        roofline["frac_of_stream_read"] = round(achieved / stream_read["GB/s"], 4)

    # ---- what the synthetic layer looks like to the Top-k: concentration per head, budgets --------
    res = step(0)
    torch.cuda.synchronize()
    conc, pos = [], 0
    for b in range(wl.batch):
        for c in range(wl.h_kv):
            row = res["scores"][pos:pos + wl.n[b]]
            top = torch.topk(row, max(1, int(0.05 * wl.n[b]))).values.sum()
            conc.append(float(top / row.sum()))
            pos += wl.n[b]
    bud = res["budgets"].cpu().numpy()
    stats = {"top5pct_score_mass_per_head": [round(c, 3) for c in conc] if len(conc) <= 16 else
             {"min": round(min(conc), 3), "median": round(float(np.median(conc)), 3), "max": round(max(conc), 3)},
             "budgets_min": int(bud.min()), "budgets_max": int(bud.max()),
             "uniform_share": [(B - wl.w * wl.h_kv) // wl.h_kv for B in wl.B] if wl.batch <= 8 else None,
             "input_set": 0}

    # ---- the oracle on the host cores: whole layers of the same workload, about 10 s ----------
    cpu = None
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info

        from oracle import adakv_oracle as O
        off = wl.tok_off
        done_tokens, layers_done, spent = 0, 0, 0.0
        while spent < 10.0 and layers_done < 64:
            q, K, V = sets[layers_done % len(sets)]
            for b in range(wl.batch):
                qd = q[b].double().cpu().numpy()
                Kd = K[off[b]:off[b + 1]].double().cpu().numpy()
                Vd = V[off[b]:off[b + 1]].float().cpu().numpy()
                c0 = time.perf_counter()
                O.compress_layer(qd, Kd, Vd, wl.n[b], wl.w, wl.pool_k, wl.B[b], wl.alpha,
                                 order="pool_then_mean" if args.pool_then_mean else "mean_then_pool")
                spent += time.perf_counter() - c0
                done_tokens += wl.n[b]
            layers_done += 1
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        cpu = {"value": round(done_tokens / spent, 1), "unit": "prefix tokens/s", "cores": threads,
               "kind": "oracle", "seconds": round(spent, 3),
               "sample": f"{layers_done} whole layer call(s) of {wl.name} (all four steps, {done_tokens} prefix "
                         f"tokens), fp64 numpy; {threads} BLAS threads for the logit matmuls, the rest "
                         "single-threaded; upcasting the inputs to fp64 is not timed"}

    out = {
        "metric": "prefix tokens compressed/sec per layer (score+allocate+select+compact)",
        "value": round(value, 1), "unit": "prefix tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": {"torch.bfloat16": "bf16", "torch.float16": "f16"}.get(str(wl.dtype), "f32"), "data": "synthetic",
        "config": {"workload": wl.name, "h_q": wl.h_q, "h_kv": wl.h_kv, "d": wl.d, "n": wl.n,
                   "w": wl.w, "pool_k": wl.pool_k, "B": wl.B, "alpha": wl.alpha, "batch": wl.batch,
                   "input_sets_rotated": len(sets),
                   "row_lse": "supplied by the caller (single sweep)" if args.row_lse else "computed (two sweeps)",
                   "order": "pool every row, then mean (Alg. 2 l.4 as printed)" if args.pool_then_mean
                   else "mean over the rows, then pool",
                   "layer_budgets": "equal" if args.pyramid is None else
                   f"pyramid over {args.sets} layers, ratio {args.pyramid}: " + str([L.num_rows_out for L in layers]),
                   "layers_in_flight": max(1, args.streams)},
        "median_ms_per_step": round(median_ms, 5) if median_ms is not None else None,
        "pipeline_hbm_frac": round(total_alg / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "pipeline_algorithmic_bytes": total_alg,
        "pipeline_traffic_bytes": step_traffic,
        "pipeline_traffic_over_algorithmic": round(step_traffic / total_alg, 3) if step_traffic else None,
        "score_mfma_tflops": round(flops / (sum(v for k, v in kernels.items() if k.startswith("score_")) * 1e-6) / 1e12, 2),
        "kernels_us": {k: round(kernels[k], 2) for k in order},
        "stream_read": stream_read, "workload_stats": stats,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
