#!/usr/bin/env python3
"""Benchmark of the DiffQKV attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload decode_32k]

A step is one pass of the whole path over one batch of synthetic input: for the decode workloads a
`diffqkv_decode` / `diffqkv_decode_paged` call (split kernel + log-sum-exp combine), for the prefill
workload a `diffqkv_prefill` call.  Inputs are resident in HBM before the timed region.  Consecutive
steps rotate through several copies of the cache at distinct addresses so that the 256 MB
last-level cache cannot serve a step from what the previous one left behind.

Prints one JSON line.  `value` is whole-job throughput: KV-cache bytes read per second (decode) or
attention TFLOP/s (prefill), from the wall clock around exactly K steps.  `roofline` is for the
dominant kernel alone: its average duration over a second pass of the same K steps in which every
launch carries a pair of HIP events attached to its own dispatch on the launch stream (the library's
experimental kernel timer); `cpu_baseline` is the float64 oracle on the host cores, for context only.

Without `--workload` the line is the headline workload (decode_32k) and carries an `also` object with
the other three attention workloads (prefill_8k, decode_4k, paged_ragged), each timed the same way
with a fixed, smaller number of steps.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
ROTATE_BYTES = 2.5e9        # keep at least this many distinct cache bytes in rotation


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=None,
                    choices=["decode_32k", "decode_4k", "paged_ragged", "prefill_8k", "decode_32k_halfk",
                             "prefill_8k_halfk", "augq_1p5b", "augq_10b"],
                    help="*_halfk: the same shapes with K heads of half width (d_qk 64, d_v 128); the last two "
                         "time the augmented-Q feed-forward of a decode step (16 tokens) at Sigma-1.5B / "
                         "Sigma-10B widths: weight bytes per second")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="default run: headline workload only")
    ap.add_argument("--top-k", type=int, default=-1,
                    help="contiguous decode workloads only: selective V-cache fetching with this top_k "
                         "(a different, smaller byte count; not the headline metric)")
    ap.add_argument("--prefill-waves", type=int, default=0, help="prefill kernel variant (experiments)")
    ap.add_argument("--chunk", type=int, default=0, help="override tokens per context split (experiments)")
    return ap.parse_args()


# (workload, steps, warm-up).  The prefill kernel needs a long warm-up: under its sustained matrix-core
# load the chip's clock first dips (launches of 1.0-1.2 ms) and takes about 35 launches to settle.
ALSO = (("prefill_8k", 50, 50), ("decode_4k", 200, 20), ("paged_ragged", 30, 10))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); nothing in it uses a second device",
              file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2501_13629_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    binding.load_library()  # fail loudly if the HIP library is not built
    binding.diffqkv_set_tuning(decode_chunk_tokens=args.chunk, prefill_waves=args.prefill_waves)
    dev = torch.device("cuda:0")
    headline = args.workload or "decode_32k"
    if headline.startswith("augq"):
        return bench_augq(args, torch, binding, inputs, dev)
    if args.top_k >= 0 and inputs.config(headline)["kind"] != "decode":
        print("bench.py: --top-k goes with the contiguous decode workloads", file=sys.stderr)
        sys.exit(2)
    line = run_workload(headline, args.steps, args.warmup, args.top_k, not args.no_cpu_baseline, torch, binding,
                        inputs, dev)
    if args.workload is None and args.top_k < 0 and not args.no_also:
        also = {}
        for name, steps, warmup in ALSO:
            r = run_workload(name, steps, warmup, -1, False, torch, binding, inputs, dev)
            also[name] = {k: r[k] for k in ("metric", "value", "unit", "steps", "warmup", "ms_per_step")}
            also[name]["roofline"] = r["roofline"]
            also[name]["config"] = r["config"]
        line["also"] = also
    print(json.dumps(line))


def run_workload(workload, steps, warmup, topk, want_cpu, torch, binding, inputs, dev):
    cfg = inputs.config(workload)
    kind = cfg["kind"]
    props = torch.cuda.get_device_properties(0)
    # ---- inputs, resident on the device ----------------------------------------------------------
    if kind == "decode":
        host = inputs.make_decode(cfg)
        kv_bytes = cfg["B"] * cfg["T"] * inputs.kv_bytes_per_token(cfg)
        if topk >= 0:  # all of K, and per query head the selected V rows plus the current token's
            kv_bytes = 2 * cfg["B"] * (cfg["T"] * cfg["n_k"] * cfg["d_qk"] +
                                       cfg["n_q"] * (min(topk, cfg["T"] - 1) + 1) * cfg["d_v"])
        cache_names = ("k", "v")
    elif kind == "paged":
        host = inputs.make_paged(cfg)
        kv_bytes = int(host["seqlens"].sum().item()) * inputs.kv_bytes_per_token(cfg)
        cache_names = ("k_pool", "v_pool")
    else:
        host = inputs.make_prefill(cfg)
        kv_bytes = 0
        cache_names = ()
    q = host["q"].to(dev)
    set_bytes = sum(host[n].numel() * host[n].element_size() for n in cache_names)
    n_sets = 1 if not cache_names else max(2, min(8, int(-(-ROTATE_BYTES // max(set_bytes, 1)))))
    sets = []
    for i in range(n_sets):
        sets.append({n: (host[n].to(dev) if i == 0 else sets[0][n].clone()) for n in cache_names})
    if kind == "paged":
        bt, sl = host["block_table"].to(dev), host["seqlens"].to(dev)
        max_T = host["max_pages"] * host["page_size"]
    if kind != "prefill":
        ws_bytes = binding.diffqkv_decode_workspace_bytes(cfg["B"], cfg["n_q"], cfg["n_k"], cfg["n_v"], cfg["d_qk"],
                                                          cfg["d_v"], binding.BF16,
                                                          cfg["T"] if kind == "decode" else max_T)
        if topk >= 0:
            ws_bytes = binding.diffqkv_decode_topk_workspace_bytes(cfg["B"], cfg["n_q"], cfg["n_k"], cfg["n_v"],
                                                                   cfg["d_qk"], cfg["d_v"], binding.BF16, cfg["T"])
        workspace = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        out = torch.empty((cfg["B"], cfg["n_q"], cfg["d_v"]), dtype=q.dtype, device=dev)
    else:
        k_dev, v_dev = host["k"].to(dev), host["v"].to(dev)
        out = torch.empty((cfg["B"], cfg["n_q"], cfg["S"], cfg["d_v"]), dtype=q.dtype, device=dev)
        S = cfg["S"]
        # two products of d_qk and d_v multiply-adds per visible (query, key) pair; masked half not counted
        flops = 2.0 * (cfg["d_qk"] + cfg["d_v"]) * cfg["B"] * cfg["n_q"] * S * (S + 1) / 2

    def step(i):
        if kind == "decode":
            s = sets[i % n_sets]
            if topk >= 0:
                binding.diffqkv_decode_topk(q, s["k"], s["v"], topk, out=out, workspace=workspace)
            else:
                binding.diffqkv_decode(q, s["k"], s["v"], out=out, workspace=workspace)
        elif kind == "paged":
            s = sets[i % n_sets]
            binding.diffqkv_decode_paged(q, s["k_pool"], s["v_pool"], bt, sl, out=out, workspace=workspace)
        else:
            binding.diffqkv_prefill(q, k_dev, v_dev, causal=True, out=out)

    # ---- warm-up, then exactly K timed steps -------------------------------------------------------
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps

    # ---- the kernels alone: the same K steps again, back to back, with the library's kernel timer on --
    # (every split / combine / prefill launch carries a pair of HIP events attached to its own dispatch
    #  on the launch stream; the pair reads the kernel's duration as rocprofv3's kernel trace does)
    binding.diffqkv_kernel_timer(True)
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    timed_ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    avg_main_us, avg_tail_us, n_timed = binding.diffqkv_kernel_timer_read()
    binding.diffqkv_kernel_timer(False)
    assert n_timed == steps, (n_timed, steps)
    if topk >= 0:  # both kernels of the top-k path count as "the kernel"
        avg_main_us, avg_tail_us = avg_main_us + avg_tail_us, 0.0

    # ---- stream-read ceiling of this machine, over the same byte count -----------------------------------
    ceiling = None
    if kind != "prefill":
        sink = torch.empty(4096, dtype=torch.float32, device=dev)
        bufs = [torch.cat([s[n].reshape(-1) for n in cache_names]) for s in sets[: min(n_sets, 4)]]
        for b in bufs:
            binding.diffqkv_probe_stream_read(b, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 5 * len(bufs)
        e0.record()
        for r in range(reps):
            binding.diffqkv_probe_stream_read(bufs[r % len(bufs)], sink)
        e1.record()
        torch.cuda.synchronize()
        ceiling = bufs[0].numel() * bufs[0].element_size() * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del bufs

    # ---- result ------------------------------------------------------------------------------------
    if kind != "prefill":
        value = kv_bytes / (ms_per_step * 1e-3) / 1e9
        metric, unit = "decode-attention achieved HBM GB/s", "GB/s"
        if topk >= 0:
            metric = "decode-attention with top-%d V fetching, algorithmic GB/s" % topk
        achieved = kv_bytes / (avg_main_us * 1e-6) / 1e9
        roof = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                "kernel": "decode_mfma_kernel (split)" if topk < 0 else "topk_scores + topk_select (both)",
                "kernel_avg_us": round(avg_main_us, 2), "combine_avg_us": round(avg_tail_us, 2),
                "kernel_timing": "HIP events attached to each dispatch, all %d steps of a second timed pass" % steps,
                "us_per_step_with_timer_on": round(timed_ms_per_step * 1e3, 2),
                "step_frac": round(value / HBM_PEAK_GBPS, 4),
                "algorithmic_bytes_per_launch": kv_bytes,
                "stream_read_ceiling_GBps": None if ceiling is None else round(ceiling, 1)}
    else:
        value = flops / (ms_per_step * 1e-3) / 1e12
        metric, unit = "causal-prefill attention TFLOP/s", "TFLOP/s"
        achieved = flops / (avg_main_us * 1e-6) / 1e12
        roof = {"bound": "mfma", "achieved": round(achieved, 1), "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / BF16_PEAK_TFLOPS, 4), "traffic": None, "kernel": "prefill kernel",
                "kernel_avg_us": round(avg_main_us, 2),
                "kernel_timing": "HIP events attached to each dispatch, all %d steps of a second timed pass" % steps,
                "us_per_step_with_timer_on": round(timed_ms_per_step * 1e3, 2),
                "step_frac": round(value / BF16_PEAK_TFLOPS, 4),
                "algorithmic_flops_per_launch": flops}
    # HBM bytes per launch come from separate rocprofv3 --pmc runs of this same command (counters cannot
    # be read from inside the process); the figure is a stored measurement, and says so
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    roof["traffic_source"] = None
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            roof["traffic"] = json.load(f).get(workload if topk < 0 else "%s_topk%d" % (workload, topk))
        if roof["traffic"] is not None:
            roof["traffic_source"] = ("stored: profiles/hbm_traffic.json, rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE "
                                      "of an earlier run of this workload, not measured in this run")

    cpu = cpu_baseline(cfg, host, kind, kv_bytes, topk) if want_cpu else None

    line = {
        "metric": metric, "value": round(value, 2), "unit": unit, "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(ms_per_step, 5), "us_per_step": round(ms_per_step * 1e3, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4) if kind != "prefill" else None,
        "config": {"workload": workload if topk < 0 else "%s, top_k=%d" % (workload, topk), **{k: v for k, v in cfg.items()
                                                 if k in ("B", "n_q", "n_k", "n_v", "d_qk", "d_v", "T", "S", "page_size")},
                   "kv_bytes_per_step": kv_bytes, "cache_sets_in_rotation": n_sets,
                   "device": props.name, "compute_units": props.multi_processor_count},
        "roofline": roof, "cpu_baseline": cpu,
    }
    del sets, q, out
    torch.cuda.empty_cache()
    return line


def bench_augq(args, torch, binding, inputs, dev):
    """The augmented-Q feed-forward of one decode step: 16 tokens, weights streamed once per step."""
    M = 16
    hidden, inter = (2048, 3072) if args.workload == "augq_1p5b" else (4096, 6144)
    host = inputs.make_augq(M, hidden, inter, "bf16", 46)
    names = ("q_in", "w_gate", "w_up", "w_down")
    wbytes = 3 * hidden * inter * 2
    n_sets = max(2, min(16, int(-(-ROTATE_BYTES // wbytes))))  # distinct weight copies: no cache reuse across steps
    sets = [[host[n].to(dev) for n in names]]
    for _ in range(n_sets - 1):
        sets.append([sets[0][0]] + [t.clone() for t in sets[0][1:]])
    out = torch.empty((M, hidden), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(M * inter * 2 + 256, dtype=torch.uint8, device=dev)

    def step(i):
        binding.diffqkv_augment_q(*sets[i % n_sets], out=out, workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    us = wall * 1e6 / args.steps
    binding.diffqkv_kernel_timer(True)
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    k0, k1, _ = binding.diffqkv_kernel_timer_read()
    binding.diffqkv_kernel_timer(False)
    avg = k0 + k1
    value = wbytes / (us * 1e-6) / 1e9
    traffic, traffic_file = None, os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            traffic = json.load(f).get(args.workload)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        a = [inputs.as_numpy(host[n]) for n in names]
        reps, t0 = 0, time.perf_counter()
        while True:
            oracle.augment_q(*a)
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= 10.0 or reps >= 1000:
                break
        cpu = {"value": round(wbytes * reps / dt / 1e9, 4), "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "the full workload, %d evaluations" % reps, "seconds": round(dt, 3)}
    print(json.dumps({
        "metric": "augmented-Q feed-forward, weight GB/s", "value": round(value, 2), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us / 1e3, 5), "us_per_step": round(us, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "M": M, "hidden": hidden, "inter": inter, "weight_bytes_per_step": wbytes,
                   "weight_sets_in_rotation": n_sets},
        "roofline": {"bound": "hbm", "achieved": round(wbytes / (avg * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(wbytes / (avg * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_source": None if traffic is None else "stored: profiles/hbm_traffic.json, rocprofv3 --pmc "
                     "FETCH_SIZE and WRITE_SIZE of an earlier run of this workload, not measured in this run",
                     "kernel": "augq_mfma_kernel<true> + <false> (both launches)", "kernel_avg_us": round(avg, 2),
                     "first_product_us": round(k0, 2), "second_product_us": round(k1, 2),
                     "algorithmic_bytes_per_launch": wbytes},
        "cpu_baseline": cpu}))


def cpu_baseline(cfg, host, kind, kv_bytes, topk=-1):
    """The float64 oracle as it stands, on the host cores, over a bounded sample of the workload."""
    import numpy as np

    import oracle
    from paper_2501_13629_amd import inputs

    a = inputs.as_numpy
    threads = oracle.num_threads()
    if kind == "decode":
        if topk >= 0:
            fn = lambda: oracle.decode_topk(a(host["q"]), a(host["k"]), a(host["v"]), topk)
        else:
            fn = lambda: oracle.decode(a(host["q"]), a(host["k"]), a(host["v"]))
        work, unit, sample = kv_bytes / 1e9, "GB/s", "the full workload, one evaluation"
    elif kind == "paged":
        n = 16  # sequences
        fn = lambda: oracle.decode_paged(a(host["q"])[:n], a(host["k_pool"]), a(host["v_pool"]),
                                         host["block_table"].numpy()[:n], host["seqlens"].numpy()[:n])
        work = int(host["seqlens"][:n].sum().item()) * inputs.kv_bytes_per_token(cfg) / 1e9
        unit, sample = "GB/s", "the first %d of %d sequences, one evaluation" % (n, cfg["B"])
    else:
        rows = np.arange(0, cfg["S"], 128, dtype=np.int32)  # every 128th query row, all heads
        fn = lambda: oracle.prefill(a(host["q"]), a(host["k"]), a(host["v"]), causal=True, rows=rows)
        work = float(sum(2.0 * (cfg["d_qk"] + cfg["d_v"]) * cfg["B"] * cfg["n_q"] * (int(i) + 1) for i in rows)) / 1e12
        unit, sample = "TFLOP/s", "every 128th query row of every head (%d rows), one evaluation" % len(rows)
    # repeat the sample until about ten seconds of CPU work have been timed (at least one evaluation)
    reps, t0 = 0, time.perf_counter()
    while True:
        fn()
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or reps >= 1000:
            break
    sample = sample.replace("one evaluation", "%d evaluation%s" % (reps, "" if reps == 1 else "s"))
    return {"value": round(work * reps / dt, 4), "unit": unit, "cores": threads, "kind": "oracle", "sample": sample,
            "seconds": round(dt, 3)}


if __name__ == "__main__":
    main()
