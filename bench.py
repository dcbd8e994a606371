#!/usr/bin/env python3
"""Benchmark of the paged-KV decode-attention hot path on one MI355X.

A step is one kv_decode_attn call (main kernel + split-KV combine) over one synthetic
batch of the chosen workload, inputs resident in HBM.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1|2|3] [--prefetch-distance k]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def log(msg):
    print(msg, file=sys.stderr, flush=True)


_EVENT_OVERHEAD_MS = None


def event_bracket_overhead(torch, pairs=200):
    """What a pair of HIP events costs by itself: the median time between two events recorded back to back on
    the launch stream with nothing between them (about 5 us on this chip).  A bracket around a kernel reads
    that much more than the kernel's own duration, so it is subtracted from every event-based kernel time."""
    global _EVENT_OVERHEAD_MS
    if _EVENT_OVERHEAD_MS is None:
        def pair():
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            b.record()
            return a, b
        for _ in range(10):
            pair()
        torch.cuda.synchronize()
        ps = [pair() for _ in range(pairs)]
        torch.cuda.synchronize()
        _EVENT_OVERHEAD_MS = sorted(a.elapsed_time(b) for a, b in ps)[pairs // 2]
    return _EVENT_OVERHEAD_MS


def timed_steps(kv, torch, cases, pd, steps, warmup):
    """W untimed + K timed steps, alternating between the cache copies.  Returns
    (ms per step by wall clock, main-kernel ms per launch by HIP events on the launch stream, less what an
    empty event bracket reads)."""
    overhead = event_bracket_overhead(torch)
    def step(i):
        c = cases[i % len(cases)]
        if "k_scale" in c:                       # 8-bit cache
            kv.kv_decode_attn_kv8(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], c["out"],
                                  c["scale"], c["k_scale"], c["v_scale"], c["num_kv_heads"], c["block_size"], pd)
        else:
            kv.kv_decode_attn(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], c["out"],
                              c["scale"], c["num_kv_heads"], c["block_size"], pd)
    for i in range(warmup):
        step(i)
    every = 4                                  # every 4th launch of the timed region carries an event pair
    kv.kv_profile_enable((steps + every - 1) // every, every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    main_ms, n = kv.kv_profile_read()
    kv.kv_profile_enable(0, 1)
    assert n == (steps + every - 1) // every
    return (t1 - t0) * 1e3 / steps, main_ms / n - overhead


def layer_stack(kv, torch, synth, dev, steps, warmup, pd, cross, layers=None):
    """Benchmark configuration 4: `layers` x (dense layer [128 x 4096].[4096 x 14336] + paged decode attention on
    that layer's own KV cache).  Returns ms per stack pass and the bytes one pass must move."""
    cfg = synth.CONFIGS[4]
    L = layers or cfg["layers"]
    seed = synth.config_seed(4)
    lens = synth.context_lengths(cfg, seed)
    cases = [synth.make_case(cfg, seed, dev, lens=lens, data_seed=seed + 1000 * l) for l in range(L)]
    x = synth.randn16((cfg["B"], cfg["gemm_k"]), "bf16", seed + 11, dev)
    # weights ~ N(0, 0.02), handed over in the library's tile-packed layout (set-up time, not timed)
    ws = [kv.pack_weights(synth.randn16((cfg["gemm_k"], cfg["gemm_n"]), "bf16", seed + 13 + l, dev) * 0.02) for l in range(L)]
    y = torch.empty((cfg["B"], cfg["gemm_n"]), dtype=torch.bfloat16, device=dev)
    outs = [torch.empty_like(c["q"]) for c in cases]
    c0 = cases[0]
    ks, vs = [c["k_cache"] for c in cases], [c["v_cache"] for c in cases]

    def step():
        kv.kv_decode_layerstack(x, ws, y, None, ks, vs, c0["block_tables"], c0["context_lens"], outs, c0["scale"],
                                c0["num_kv_heads"], c0["block_size"], pd, cross)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    kvb = synth.kv_bytes(lens, cfg["Hkv"], cfg["d"]) * L
    wb = cfg["gemm_k"] * cfg["gemm_n"] * 2 * L
    return ms, kvb, wb, cfg, L


def fetch_ceiling(kv, torch, cases, kvb, steps=40, warmup=8):
    """The memory system's rate for the kernel's own access pattern: the fetch stream of the attention kernel
    with its arithmetic left out (kv_decode_fetch_probe), beside the attention kernel itself, for a grid of
    (waves per compute unit, prefetch distance); main-kernel microseconds from the library's HIP events."""
    def timed(fn, pd):
        def step(i):
            c = cases[i % len(cases)]
            fn(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], c["out"], c["scale"],
               c["num_kv_heads"], c["block_size"], pd)
        for i in range(warmup):
            step(i)
        kv.kv_profile_enable(steps, 1)
        torch.cuda.synchronize()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        ms, n = kv.kv_profile_read()
        kv.kv_profile_enable(0, 1)
        return ms / n * 1e3
    rows = []
    d = cases[0]["q"].shape[2]
    try:
        for waves, pd in ((2, 2), (2, 4), (4, 1), (4, 2), (6, 0), (6, 1), (6, 2), (8, 1), (12, 0), (16, 0)):
            kv.kv_decode_set_waves_per_cu(waves)
            probe_us, attn_us = timed(kv.kv_decode_fetch_probe, pd), timed(kv.kv_decode_attn, pd)
            rows.append({"waves_per_cu": kv.kv_decode_get_waves_per_cu(pd, d), "prefetch_distance": pd,
                         "fetch_only_us": round(probe_us, 1), "fetch_only_GBps": round(kvb / probe_us / 1e3, 0),
                         "attention_us": round(attn_us, 1), "attention_GBps": round(kvb / attn_us / 1e3, 0)})
            log(f"[bench] {rows[-1]}")
    finally:
        kv.kv_decode_set_waves_per_cu(0)
    return rows


HEATMAP_MODELS = {               # attention shapes of the paper's four models (Section 4.1), head_dim 128, 16-token blocks
    "mha_32q_32kv": (32, 32), "gqa_32q_8kv": (32, 8), "gqa_28q_4kv": (28, 4), "gqa_40q_8kv": (40, 8),
}


def worker_timeline(kv, torch, cases, pd, launches=8):
    """Where the main kernel's time goes inside a launch: every persistent worker reports the 100 MHz clock at
    entry, after locating its range and at exit (kv_decode_set_worker_trace).  Percentiles over the workers of
    the last launch, in microseconds after the first worker's entry."""
    import numpy as np
    cfg_d = cases[0]["q"].shape[2]
    trace = torch.zeros((4096, 4), dtype=torch.int64, device=cases[0]["q"].device)
    kv.kv_decode_set_worker_trace(trace)
    try:
        for i in range(launches):
            c = cases[i % len(cases)]
            kv.kv_decode_attn(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], c["out"],
                              c["scale"], c["num_kv_heads"], c["block_size"], pd)
        torch.cuda.synchronize()
    finally:
        kv.kv_decode_set_worker_trace(None)
    t = trace.cpu().numpy()
    t = t[t[:, 3] > 0]                         # workers that had a range
    xcd, t[:, 3] = t[:, 3] >> 32, t[:, 3] & 0xffffffff
    t0 = t[:, 0].min()
    us = lambda col: (t[:, col] - t0) / 100.0
    pct = lambda a: {f"p{q}": round(float(np.percentile(a, q)), 2) for q in (0, 10, 50, 90, 100)}
    return {"workers": int(len(t)), "waves_per_cu": kv.kv_decode_get_waves_per_cu(pd, cfg_d),
            "tiles_per_worker": [int(t[:, 3].min()), int(t[:, 3].max())],
            "entry_us": pct(us(0)), "range_located_us": pct(us(1)), "exit_us": pct(us(2)),
            "busy_us": pct((t[:, 2] - t[:, 1]) / 100.0),
            "mean_exit_us_by_xcd": {int(x): round(float(us(2)[xcd == x].mean()), 2) for x in np.unique(xcd)}}


def heatmap(kv, torch, synth, dev, pd_on, steps=20, warmup=4):
    """Synthetic counterpart of the paper's batch x sequence-length sweep (Section 4.3, Figure 4): main-kernel time
    with the look-ahead on and off for every (model shape, batch, context) cell; equal context lengths per cell."""
    rows = []
    for name, (Hq, Hkv) in HEATMAP_MODELS.items():
        for B in (1, 4, 16, 64, 128):
            for ctx in (1024, 2560, 4608, 8704):             # 512 input tokens + 512 .. 8192 generated
                cfg = dict(Hq=Hq, Hkv=Hkv, d=128, bs=16, dtype="bf16")
                cases = []
                for i in range(2):
                    c = synth.make_case(cfg, synth.BASE_SEED + 17 * i, dev, lens=[ctx] * B)
                    c["out"] = torch.empty_like(c["q"])
                    cases.append(c)
                kvb = synth.kv_bytes([ctx] * B, Hkv, 128)
                t = {}
                for label, pd in (("on", pd_on), ("off", 0)):
                    def step(i):
                        c = cases[i % 2]
                        kv.kv_decode_attn(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"],
                                          c["out"], c["scale"], Hkv, 16, pd)
                    for i in range(warmup):
                        step(i)
                    kv.kv_profile_enable(steps, 1)
                    torch.cuda.synchronize()
                    for i in range(steps):
                        step(i)
                    torch.cuda.synchronize()
                    ms, n = kv.kv_profile_read()
                    kv.kv_profile_enable(0, 1)
                    t[label] = ms / n
                rows.append({"model": name, "batch": B, "context": ctx, "kv_bytes": kvb, "on_us": t["on"] * 1e3,
                             "off_us": t["off"] * 1e3, "speedup": t["off"] / t["on"], "on_GBps": kvb / t["on"] / 1e6})
                del cases
                torch.cuda.empty_cache()
        log(f"[bench] heat-map {name} done")
    return rows


def cpu_baseline(oracle, synth, case, cfg, budget_s=20.0, min_wall_s=1.5):
    """The oracle as it stands, timed on the host cores over whole sequences of the same batch: a sample sized
    to at most `budget_s` of wall time, repeated until about `min_wall_s` have passed (tens of core-seconds)."""
    import numpy as np
    bits = dict(q=oracle.bits_of(case["q"]), k=oracle.bits_of(case["k_cache"]), v=oracle.bits_of(case["v_cache"]),
                bt=case["block_tables"].cpu().numpy(), cl=case["context_lens"].cpu().numpy())
    lens = case["lens"]
    Hq = cfg["Hq"]

    def run(pairs):
        t0 = time.perf_counter()
        oracle.paged_attention(bits["q"], bits["k"], bits["v"], bits["bt"], bits["cl"], case["scale"], case["dtype"], pairs)
        return time.perf_counter() - t0

    # a first short probe sizes the sample to the time budget
    probe = np.array([(0, h) for h in range(min(Hq, 8))], np.int32)
    dt = run(probe)
    rate = max(int(lens[0]), 1) * len(probe) / max(dt, 1e-6)          # (token, q-head) pairs per second, few threads busy
    total_work = int(lens.sum()) * Hq
    nseq = len(lens)
    if total_work / rate > budget_s:
        nseq = max(1, int(nseq * budget_s * rate / total_work))
    pairs = np.array([(b, h) for b in range(nseq) for h in range(Hq)], np.int32)
    wall, reps = 0.0, 0
    while wall < min_wall_s and reps < 50:
        wall += run(pairs)
        reps += 1
    kvb = synth.kv_bytes(lens[:nseq], cfg["Hkv"], cfg["d"])
    threads = oracle.oracle_threads()
    return {"value": kvb * reps / wall / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"first {nseq} of {len(lens)} sequences, all {Hq} query heads ({kvb / 1e6:.1f} MB of KV), "
                      f"{reps} passes in {wall:.2f} s on {threads} threads",
            "tokens_per_s": nseq * reps / wall}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=1, choices=[1, 2, 3])
    ap.add_argument("--prefetch-distance", type=int, default=None)
    ap.add_argument("--waves-per-cu", type=int, default=0, help="persistent waves per compute unit (0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the prefetch-off leg and the other workloads")
    ap.add_argument("--layer-stack-only", type=int, default=0, metavar="LAYERS",
                    help="run only the layer stack with this many layers and print its record (profiling aid)")
    ap.add_argument("--cross-layer-touch", type=int, default=0)
    ap.add_argument("--heatmap", action="store_true",
                    help="print the on/off sweep over model shape x batch x context length and exit")
    ap.add_argument("--kv8", action="store_true",
                    help="time the 8-bit (FP8 E4M3) KV cache entry point on the workload instead (with --no-extra: for "
                         "profiler runs of that kernel); GB/s then counts the 8-bit bytes")
    ap.add_argument("--worker-timeline", action="store_true",
                    help="print the per-worker entry / exit times of one launch of the main kernel and exit")
    ap.add_argument("--l2-touch", type=int, default=0, metavar="TILES",
                    help="comparison mode: with --prefetch-distance 0, a second wave per worker touches this many tiles "
                         "per group into L2 ahead of it (the paper's mechanism in place of the LDS ring)")
    ap.add_argument("--two-phase", action="store_true",
                    help="comparison variant: the two-phase kernel form (all logits of a chunk, then the V tiles)")
    ap.add_argument("--fetch-ceiling", action="store_true",
                    help="time the attention kernel's fetch stream without its arithmetic beside the kernel itself "
                         "over a grid of occupancies and prefetch distances, print the table and exit")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run plain 1 GiB device copies, so a counter run sees a copy kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; run with --gpus 1 "
              "(the path shards by kv head or by sequence with no exchange step)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2504_06319_amd as kv
    from paper_2504_06319_amd import synth

    if not os.path.exists(kv.library_path()):
        from paper_2504_06319_amd.build import build_library
        build_library()
    kv.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.waves_per_cu:
        kv.kv_decode_set_waves_per_cu(args.waves_per_cu)
    if args.l2_touch:
        kv.kv_decode_set_l2_touch(args.l2_touch)
    if args.two_phase:
        kv.kv_decode_set_variant(kv.KV_VARIANT_TWO_PHASE)

    def make_cases(index, copies=2, kv8=False):
        cfg = synth.CONFIGS[index]
        out = []
        make = synth.make_case_kv8 if kv8 else synth.make_case
        for i in range(copies):      # distinct cache copies so no launch re-reads what the last one left in cache
            c = make(cfg, synth.config_seed(index) + 100000 * i, dev, lens=None if i == 0 else out[0]["lens"])
            c["out"] = torch.empty_like(c["q"])
            out.append(c)
        return cfg, out

    def measure(index, pd, steps, warmup, kv8=False):
        cfg, cases = make_cases(index, kv8=kv8)
        kvb = synth.kv_bytes(cases[0]["lens"], cfg["Hkv"], cfg["d"], 1 if kv8 else 2)
        ms, main_ms = timed_steps(kv, torch, cases, pd, steps, warmup)
        return cfg, cases, kvb, ms, main_ms

    if args.traffic_calibration:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device=dev)      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    pd_on = args.prefetch_distance if args.prefetch_distance is not None else (1 if args.kv8 else 2)
    if args.heatmap:
        print(json.dumps({"heatmap": heatmap(kv, torch, synth, dev, pd_on), "prefetch_distance": pd_on,
                          "waves_per_cu": kv.kv_decode_get_waves_per_cu(pd_on, 128)}), flush=True)
        return
    if args.worker_timeline:
        cfg, cases = make_cases(args.workload)
        print(json.dumps({"workload": cfg["name"], "prefetch_distance": pd_on,
                          "worker_timeline": worker_timeline(kv, torch, cases, pd_on)}), flush=True)
        return
    if args.fetch_ceiling:
        cfg, cases = make_cases(args.workload)
        kvb = synth.kv_bytes(cases[0]["lens"], cfg["Hkv"], cfg["d"])
        print(json.dumps({"workload": cfg["name"], "kv_bytes_per_launch": kvb,
                          "fetch_ceiling": fetch_ceiling(kv, torch, cases, kvb)}), flush=True)
        return
    if args.layer_stack_only:
        lms, lkvb, lwb, lcfg, L = layer_stack(kv, torch, synth, dev, args.steps, args.warmup, pd_on, args.cross_layer_touch,
                                              layers=args.layer_stack_only)
        print(json.dumps({"workload": lcfg["name"], "layers": L, "ms_per_pass": lms, "tokens_per_s": lcfg["B"] / (lms * 1e-3),
                          "GB_per_s": (lkvb + lwb) / (lms * 1e-3) / 1e9, "prefetch_distance": pd_on,
                          "cross_layer_touch": args.cross_layer_touch}), flush=True)
        return
    log(f"[bench] workload {args.workload} prefetch_distance {pd_on}")
    cfg, cases, kvb, ms, main_ms = measure(args.workload, pd_on, args.steps, args.warmup, kv8=args.kv8)
    value = kvb / (ms * 1e-3) / 1e9
    achieved = kvb / (main_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{cfg['name']}.json")
    if os.path.exists(tpath) and not args.kv8:
        with open(tpath) as f:
            traffic = json.load(f).get("traffic_bytes_per_launch")
    result = {
        "metric": "decode-attn effective KV GB/s (% of HBM peak), prefetch on vs off; tokens/s",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"] + (" (q, out) / fp8_e4m3 (KV cache)" if args.kv8 else ""), "data": "synthetic",
        "config": {"workload": cfg["name"], "batch": cfg["B"], "q_heads": cfg["Hq"], "kv_heads": cfg["Hkv"],
                   "head_dim": cfg["d"], "block_size": cfg["bs"],
                   "context_lens": "fixed" if "lens" in cfg else f"uniform{list(cfg['len_range'])}",
                   "kv_bytes_per_step": kvb, "prefetch_distance": pd_on,
                   "waves_per_cu": (kv.kv_decode_get_waves_per_cu_kv8(pd_on, cfg["d"]) if args.kv8 else
                                    kv.kv_decode_get_waves_per_cu_for(pd_on, cfg["d"], cfg["Hq"] // cfg["Hkv"])),
                   **({"l2_touch_tiles": args.l2_touch} if args.l2_touch and pd_on == 0 and not args.kv8 else {}),
                   **({"variant": "two-phase"} if args.two_phase and not args.kv8 else {})},
        "pct_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        "tokens_per_s": cfg["B"] / (ms * 1e-3),
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "attn_mfma_kernel (main attention kernel)", "kernel_ms": main_ms,
                     "kernel_ms_event_bracket": main_ms + event_bracket_overhead(torch),
                     "event_bracket_overhead_ms": event_bracket_overhead(torch),
                     "algorithmic_bytes_per_launch": kvb},
    }
    log(f"[bench] on: {ms:.4f} ms/step, {value:.0f} GB/s; main kernel {main_ms:.4f} ms")

    if args.kv8:
        result["config"]["waves_per_cu"] = kv.kv_decode_get_waves_per_cu_kv8(pd_on, cfg["d"])
        result["roofline"]["kernel"] = "attn_kv8_kernel (main attention kernel, 8-bit cache)"
        print(json.dumps(result), flush=True)
        return
    if not args.no_extra:
        _, _, _, ms0, main0 = measure(args.workload, 0, args.steps, args.warmup)
        result["prefetch_off"] = {"prefetch_distance": 0, "waves_per_cu": kv.kv_decode_get_waves_per_cu(0, cfg["d"]),
                                  "ms_per_step": ms0, "value": kvb / (ms0 * 1e-3) / 1e9,
                                  "kernel_ms": main0, "speedup_on_vs_off": ms0 / ms}
        log(f"[bench] off: {ms0:.4f} ms/step")
        # The two legs above each run at the occupancy the library picks for them (few waves with look-ahead,
        # many without).  The same comparison at EQUAL occupancy: with two waves per compute unit occupancy
        # cannot hide the HBM latency (the regime of the paper's baseline kernel, Table 1) and the look-ahead
        # does; with four or six it can, and the look-ahead adds nothing.
        low = {}
        for wpc in (2, 4, 6):
            kv.kv_decode_set_waves_per_cu(wpc)
            _, _, _, l_on, lk_on = measure(args.workload, pd_on, max(10, args.steps // 2), max(5, args.warmup // 2))
            _, _, _, l_off, lk_off = measure(args.workload, 0, max(10, args.steps // 2), max(5, args.warmup // 2))
            low[f"waves_per_cu_{wpc}"] = {"on_ms_per_step": l_on, "off_ms_per_step": l_off, "on_kernel_ms": lk_on,
                                         "off_kernel_ms": lk_off, "kernel_speedup_on_vs_off": lk_off / lk_on}
            log(f"[bench] waves/CU {wpc}: on {lk_on:.4f} ms, off {lk_off:.4f} ms kernel")
        kv.kv_decode_set_waves_per_cu(args.waves_per_cu)
        result["prefetch_on_vs_off_equal_occupancy"] = low
        others = {}
        for idx in (1, 2, 3):
            if idx == args.workload:
                continue
            torch.cuda.empty_cache()
            ocfg, _, okvb, oms, omain = measure(idx, pd_on, max(10, args.steps // 2), max(5, args.warmup // 2))
            _, _, _, oms0, _ = measure(idx, 0, max(10, args.steps // 2), max(5, args.warmup // 2))
            others[ocfg["name"]] = {"value": okvb / (oms * 1e-3) / 1e9, "unit": "GB/s", "ms_per_step": oms,
                                    "pct_hbm_peak": 100.0 * okvb / (oms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                    "kernel_ms": omain, "prefetch_off_ms_per_step": oms0,
                                    "tokens_per_s": ocfg["B"] / (oms * 1e-3)}
            log(f"[bench] {ocfg['name']}: on {oms:.4f} ms, off {oms0:.4f} ms")
        result["other_workloads"] = others
        # the same workloads on an 8-bit (FP8 E4M3) KV cache: half the bytes per token; GB/s counts the 8-bit bytes
        kv8 = {}
        for idx in (1, 2, 3):
            torch.cuda.empty_cache()
            kcfg, _, kkvb, kms, kmain = measure(idx, 1, max(10, args.steps // 2), max(5, args.warmup // 2), kv8=True)
            _, _, _, kms0, kmain0 = measure(idx, 0, max(10, args.steps // 2), max(5, args.warmup // 2), kv8=True)
            kv8[kcfg["name"]] = {"prefetch_distance": 1, "waves_per_cu": kv.kv_decode_get_waves_per_cu_kv8(1, kcfg["d"]),
                                 "kv_bytes_per_step": kkvb, "ms_per_step": kms, "value": kkvb / (kms * 1e-3) / 1e9,
                                 "unit": "GB/s", "pct_hbm_peak": 100.0 * kkvb / (kms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                 "kernel_ms": kmain, "tokens_per_s": kcfg["B"] / (kms * 1e-3),
                                 "prefetch_off_ms_per_step": kms0, "prefetch_off_kernel_ms": kmain0}
            log(f"[bench] {kcfg['name']} 8-bit cache: on {kms:.4f} ms, off {kms0:.4f} ms")
        result["kv8_cache"] = kv8
        # layer stack (configuration 4): tokens/s of 32 x (dense layer + attention), prefetch on / off, cross-layer touch
        del cases
        torch.cuda.empty_cache()
        ls = {}
        for name, pd_, cross in (("on", pd_on, 0), ("on_cross_layer_touch", pd_on, 1), ("off", 0, 0)):
            lms, lkvb, lwb, lcfg, L = layer_stack(kv, torch, synth, dev, max(3, args.steps // 20), 2, pd_, cross)
            torch.cuda.empty_cache()
            ls[name] = {"ms_per_pass": lms, "tokens_per_s": lcfg["B"] / (lms * 1e-3), "GB_per_s": (lkvb + lwb) / (lms * 1e-3) / 1e9,
                        "pct_hbm_peak": 100.0 * (lkvb + lwb) / (lms * 1e-3) / 1e9 / HBM_PEAK_GBS}
            log(f"[bench] layer stack {name}: {lms:.3f} ms/pass, {lcfg['B'] / (lms * 1e-3):.0f} tokens/s")
        ls["layers"] = L
        ls["kv_bytes_per_pass"] = lkvb
        ls["weight_bytes_per_pass"] = lwb
        result["layer_stack"] = ls
        cfg, cases = make_cases(args.workload, copies=1)

    if not args.no_cpu_baseline:
        import oracle
        torch.cuda.empty_cache()
        result["cpu_baseline"] = cpu_baseline(oracle, synth, cases[0], cfg)
        log(f"[bench] cpu baseline: {result['cpu_baseline']}")

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
