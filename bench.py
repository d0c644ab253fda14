#!/usr/bin/env python3
"""Benchmark of the DynamicKV prefill-compression hot path on one MI355X.

A step = one pass of Algorithm 1's layer loop over one synthetic batch: for every layer score (two sweeps over
K), select, gather, and the progressive update every `interval` layers.  Three schedules of the same calls are
timed (identical results, tested): `value` is the grouped one (one call per stage for as many layers as a call
takes: the caller holds Q_win, K and V of those layers), `value_layer_by_layer` is Algorithm 1's own order (one
call per stage and layer) and `value_group_interval` issues the layers of one update interval together.
All inputs are resident in HBM before the timed region.  Prints ONE JSON line: context tokens compressed per
second, the roofline of the score step (both sweeps and their two small kernels, K counted ONCE; timed live with
HIP events attached to every launch) with the per-kernel figures beside it, and the CPU oracle timed on a
bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def _cpu_baseline(cfg, host_layers, target_s=12.0):
    """The oracle as it stands on the first layers of the workload (whole update intervals), sized by a
    one-interval pilot so that the measured run takes about `target_s` seconds of CPU time."""
    from oracle import dkv_oracle as O
    cu = cfg.cu_seqlens

    def run(n_layers):
        t0 = time.perf_counter()
        for s in range(cfg.n_seqs):
            layers = [(d["q_win"][s], d["k"][:, cu[s]:cu[s + 1]], d["v"][:, cu[s]:cu[s + 1]])
                      for d in host_layers[:n_layers]]
            O.compress(layers, cfg.L, cfg.w, cfg.P, cfg.layer_max, cfg.mean_budget, cfg.interval)
        return time.perf_counter() - t0

    pilot = run(cfg.interval)
    blocks = max(1, min(len(host_layers) // cfg.interval, int(target_s / max(pilot, 1e-3))))
    n_layers = blocks * cfg.interval
    dt = run(n_layers) if blocks > 1 else pilot
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    tokens_per_s = cfg.total_tokens / (dt * cfg.L / n_layers)
    return {"value": tokens_per_s, "unit": "context tokens/s", "cores": cores, "kind": "oracle",
            "sample": "first %d of %d layers of the same workload (scoring, selection, gather, %d progressive "
                      "update(s)), %.1f s of CPU time, scaled by L/%d" % (n_layers, cfg.L, blocks, dt, n_layers)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the clocks of an idle GPU take some 10-20 ms of load to settle: the defaults warm up for that long
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--settle-ms", type=float, default=20.0,
                    help="untimed load before the warm-up passes, for the clocks of an idle GPU to settle")
    ap.add_argument("--workload", default="mistral_7b_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--group", type=int, default=0,
                    help="layers whose scoring, selection and compaction are issued together (0: as many whole update intervals as one call takes, "
                         "1: layer by layer as in Algorithm 1)")
    ap.add_argument("--overlap", action="store_true",
                    help="select/gather/rebalance of layer l on a second stream, next to the scoring of layer l+1")
    ap.add_argument("--main-only", action="store_true",
                    help="skip the side measurements (single-sweep scoring, decode attention): under a profiler the "
                         "per-kernel averages then cover the timed loop alone")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device copies (a kernel of known traffic, to scale profiler counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures ONE GPU (the path has no cross-GPU step); run with --gpus 1")

    import torch
    from paper_2412_14838_amd import dkv, workloads as W
    from paper_2412_14838_amd.pipeline import Compressor, default_group, to_device

    dkv.load()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    cfg = W.all_configs()[args.workload]
    workers = min(16, len(os.sched_getaffinity(0)))
    dev, host_sample = [], []
    with cf.ThreadPoolExecutor(max_workers=workers) as ex:
        for l, data in enumerate(ex.map(lambda l: W.make_layer(cfg, l), range(cfg.L))):
            dev.append(to_device(cfg, data))
            if not args.no_cpu_baseline and (l + 1) * cfg.Hkv * cfg.total_tokens * cfg.d * 8 < 12e9:
                host_sample.append(data)
    torch.cuda.synchronize()

    # default: as many whole update intervals as one call takes (all layers, for the configurations at hand)
    group = args.group if args.group > 0 else default_group(cfg)
    d, T = cfg.d, cfg.total_tokens
    layers = [(x["q_win"], x["k"], x["v"]) for x in dev]

    # ---- throughput: the whole loop as one HIP graph, K replays between two synchronisations
    def time_schedule(g, steps, warmup):
        c = Compressor(cfg, group=g)
        for _ in range(max(min(warmup, 3), 1)):
            c.run(layers)
        torch.cuda.synchronize()
        graph = c.capture(layers, overlap=args.overlap)
        # the GPU has idled through set-up and capture: give its clocks `--settle-ms` of load to come up (untimed,
        # reported in the JSON line), then the warm-up passes in the form that is timed
        t_settle = time.perf_counter() + args.settle_ms * 1e-3
        while time.perf_counter() < t_settle:
            graph.replay()
            torch.cuda.synchronize()
        for _ in range(max(warmup, 1)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        return c, (time.perf_counter() - t0) * 1e3 / steps

    comp, ms_per_step = time_schedule(group, args.steps, args.warmup)
    desc, cu, ws = comp.desc, comp.cu, comp.ws
    st, sh = d, T * d
    # the other schedules of the same calls: Algorithm 1's own order (one call per stage and layer) and one update
    # interval per call; fewer replays (each is reported beside `value`, never as `value`)
    other = {}
    if not args.main_only:
        for name, g in (("layer_by_layer", 1), ("group_interval", cfg.interval)):
            if g == group:
                other[name] = ms_per_step
                continue
            c2, ms2 = time_schedule(g, max(args.steps // 2, 5), max(args.warmup // 2, 2))
            other[name] = ms2
            del c2
            torch.cuda.empty_cache()

    # ---- per-kernel durations: the same K steps launched eagerly inside a profiling session of the library:
    # every launch carries its own start/stop HIP event pair on the launch stream (events cannot be read back
    # from inside a replayed graph), so each figure is the kernel's own duration, launch gaps excluded.
    launches_per_step = 5 * cfg.L + 7 * (cfg.L // cfg.interval)     # upper bound (layer by layer)
    capacity = launches_per_step * args.steps + 16
    dkv.dkv_profile_begin(capacity)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        comp.run(layers)
    enqueue_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    torch.cuda.synchronize()
    records = dkv.dkv_profile_end(capacity)
    kernel_us, kernel_n = {}, {}
    for name, us in records:
        kernel_us[name] = kernel_us.get(name, 0.0) + us
        kernel_n[name] = kernel_n.get(name, 0) + 1
    kernel_us_per_launch = {n: kernel_us[n] / kernel_n[n] for n in kernel_us}
    kernel_ms_per_step = {n: kernel_us[n] / 1e3 / args.steps for n in kernel_us}

    # ---- roofline of the score step (Eq. 1-2): all kernels of the step - statistics sweep, merge, emit sweep, border
    # fix - against the ALGORITHMIC bytes of the step, K counted once although both sweeps read it. Units: one launch
    # of the step covers `layers_per_launch` layers.
    elt = 2 if cfg.dtype == "bf16" else 4
    k_bytes = cfg.Hkv * T * d * elt                 # every key row read once
    q_bytes = cfg.n_seqs * cfg.Hq * cfg.w * d * elt
    a_bytes = cfg.Hkv * T * 4                       # pooled fp32 scores written
    step_kernels = [n for n in ("score_stats", "score_merge", "score_emit", "score_borders") if n in kernel_us]
    layers_per_launch = cfg.L * args.steps / kernel_n["score_emit"]
    step_us_per_launch = sum(kernel_us[n] for n in step_kernels) / kernel_n["score_emit"]
    step_bytes_per_layer = k_bytes + q_bytes + a_bytes
    step_bytes_per_launch = step_bytes_per_layer * layers_per_launch
    achieved = step_bytes_per_launch / (step_us_per_launch * 1e-6) / 1e9
    flops_per_sweep = 2.0 * cfg.Hq * cfg.w * T * d
    mfma_tflops = 2 * flops_per_sweep * layers_per_launch / (step_us_per_launch * 1e-6) / 1e12
    # per kernel: its own algorithmic bytes (each sweep reads K once) over its own duration
    alg_layer = {"score_stats": k_bytes + q_bytes, "score_emit": k_bytes + q_bytes + a_bytes}
    kernels = {}
    traffic_file = {}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic_file = json.load(open(tpath)).get(cfg.name, {})
        except Exception:
            traffic_file = {}
    for n in ("score_stats", "score_emit"):
        us = kernel_us[n] / kernel_n[n]
        lpl = cfg.L * args.steps / kernel_n[n]
        gbs = alg_layer[n] * lpl / (us * 1e-6) / 1e9
        kernels[n] = {"us_per_launch": us, "layers_per_launch": lpl, "bytes_per_launch": alg_layer[n] * lpl,
                      "achieved_GBs": gbs, "hbm_frac": gbs / HBM_PEAK_GBS,
                      "mfma_frac": flops_per_sweep * lpl / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                      "traffic": traffic_file.get(n, {}).get("total_bytes")}
    # counter traffic of the whole step per launch, from the committed profile (made with the grouped schedule)
    traffic = None
    if all(traffic_file.get(n, {}).get("total_bytes") for n in ("score_stats", "score_emit")) and group == default_group(cfg):
        traffic = sum(traffic_file[n]["total_bytes"] for n in traffic_file if n.startswith("score_"))
    hbm_frac, mfma_frac = achieved / HBM_PEAK_GBS, mfma_tflops / MFMA_BF16_PEAK_TFLOPS
    roofline = {"bound": "hbm", "kernel": "score step: " + " + ".join(step_kernels) + " (K counted once)",
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac, "traffic": traffic,
                "traffic_source": "profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                                  "committed; NOT measured in this run",
                "traffic_over_algorithmic": traffic / step_bytes_per_launch if traffic else None,
                "bytes_per_launch": step_bytes_per_launch, "us_per_launch": step_us_per_launch,
                "us_per_layer": step_us_per_launch / layers_per_launch,
                "layers_per_launch": layers_per_launch, "bytes_per_layer": step_bytes_per_layer,
                "mfma_tflops": mfma_tflops, "mfma_frac": mfma_frac, "mfma_peak_tflops": MFMA_BF16_PEAK_TFLOPS,
                "nearer_roofline": "hbm" if hbm_frac >= mfma_frac else "mfma",
                "kernels": kernels}

    if not args.main_only:
        # ---- the single-sweep variant (row normalisers supplied, as a prefill attention kernel would): reported
        # beside the main figure, never part of `value`. The normalisers come from the library's own statistics.
        lse_all = torch.empty((cfg.L, cfg.n_seqs, cfg.Hq, cfg.w), dtype=torch.float32, device="cuda")
        scratch_scores = torch.empty_like(comp.scores[0])
        for l, (q, k, v) in enumerate(layers):
            dkv.dkv_score_window_stats(comp.desc, q, k, d, T * d, comp.cu, scratch_scores, T, comp.ws)
            comp.row_lse(lse_all[l])
        torch.cuda.synchronize()
        dkv.dkv_profile_begin(cfg.L * args.steps + 16)
        for _ in range(args.steps):                      # `group` layers per call, as in the timed loop
            for l0 in range(0, cfg.L, group):
                part = layers[l0:l0 + group]
                comp.score_layers_from_lse(l0, [x[0] for x in part], [x[1] for x in part],
                                           [lse_all[l0 + i] for i in range(len(part))])
        torch.cuda.synchronize()
        rec = [us for name, us in dkv.dkv_profile_end(cfg.L * args.steps + 16) if name in ("score_emit", "score_merge")]
        single_us = sum(rec) / max(args.steps * cfg.L, 1)
        roofline["single_sweep_lse"] = {"us_per_layer": single_us, "layers_per_call": group,
                                        "hbm_frac": step_bytes_per_layer / (single_us * 1e-6) / 1e9 / HBM_PEAK_GBS}

        # ---- decode attention of one new token per sequence over the final compressed cache, all layers (reported
        # beside the main figure, not part of `value`)
        q_new = torch.randn((cfg.n_seqs, cfg.Hq, d), device="cuda").to(comp.tdtype)
        dec_out = torch.empty((cfg.n_seqs, cfg.Hq, d), dtype=torch.float32, device="cuda")
        for l in range(cfg.L):
            comp.decode_attention(l, q_new, dec_out)
        torch.cuda.synchronize()
        dkv.dkv_profile_begin(2 * cfg.L * args.steps + 16)
        for _ in range(args.steps):
            for l in range(cfg.L):
                comp.decode_attention(l, q_new, dec_out)
        torch.cuda.synchronize()
        rec = [us for name, us in dkv.dkv_profile_end(2 * cfg.L * args.steps + 16) if name == "decode"]
        dec_us = sum(rec) / max(args.steps * cfg.L, 1)                       # both kernels of a layer
        counts_h = comp.counts.cpu().numpy()
        rows = sum(min(cfg.w, S) * cfg.L + int(counts_h[q].sum()) for q, S in enumerate(cfg.seqlens))
        dec_bytes = rows * cfg.Hkv * d * elt * 2 / cfg.L                      # K and V rows read per layer
        roofline["decode_attention"] = {"us_per_layer": dec_us, "cache_bytes_per_layer": dec_bytes,
                                        "hbm_frac": dec_bytes / (dec_us * 1e-6) / 1e9 / HBM_PEAK_GBS}
        # the same with the layers of a call in one launch (up to 32): the kernels without the per-layer launch latency
        n_call = min(cfg.L, dkv.DKV_MAX_SELECT_LAYERS)
        q_all = torch.randn((n_call, cfg.n_seqs, cfg.Hq, d), device="cuda").to(comp.tdtype)
        out_all = torch.empty((n_call, cfg.n_seqs, cfg.Hq, d), dtype=torch.float32, device="cuda")
        for _ in range(3):
            comp.decode_attention_layers(0, n_call, q_all, out_all)
        torch.cuda.synchronize()
        dkv.dkv_profile_begin(2 * args.steps + 16)
        for _ in range(args.steps):
            comp.decode_attention_layers(0, n_call, q_all, out_all)
        torch.cuda.synchronize()
        rec = [us for name, us in dkv.dkv_profile_end(2 * args.steps + 16) if name == "decode"]
        call_us = sum(rec) / max(args.steps, 1)
        roofline["decode_attention"]["layers_in_one_call"] = {
            "layers": n_call, "us_per_call": call_us, "us_per_layer": call_us / n_call,
            "hbm_frac": dec_bytes * n_call / (call_us * 1e-6) / 1e9 / HBM_PEAK_GBS}

    out = {"metric": "context tokens compressed/s (all layers)", "value": T / (ms_per_step * 1e-3),
           "unit": "context tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": cfg.dtype, "data": "synthetic", "streams": 2 if args.overlap else 1, "layers_per_call": group, "settle_ms": args.settle_ms,
           "schedule": ("layer by layer (Algorithm 1's order)" if group == 1 else
                        "grouped: one call per stage for %d layers; the caller holds Q_win, K, V of those layers "
                        "(results identical to layer by layer)" % group),
           "config": {"workload": cfg.name, "schedule_layers_per_call": group, "layers": cfg.L, "q_heads": cfg.Hq, "kv_heads": cfg.Hkv, "head_dim": d,
                      "context": list(cfg.seqlens), "window": cfg.w, "pool": cfg.P, "mean_budget": cfg.mean_budget,
                      "layer_max": cfg.layer_max, "interval": cfg.interval},
           "roofline": roofline,
           "kernel_us_per_launch": kernel_us_per_launch, "kernel_ms_per_step": kernel_ms_per_step,
           "kernel_ms_per_step_total": sum(kernel_ms_per_step.values())}
    out["eager_enqueue_ms_per_step"] = enqueue_ms
    for name, ms in other.items():
        out["ms_per_step_" + name] = ms
        out["value_" + name] = T / (ms * 1e-3)
    if args.copy_calibration:
        x = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
        del x, y
    if host_sample:
        out["cpu_baseline"] = _cpu_baseline(cfg, host_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
