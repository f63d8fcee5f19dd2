#!/usr/bin/env python3
"""Benchmark of the WeightedKV decode step on one MI355X.

A "step" is one generated token through the whole hot path: for the default
workload (the 32-layer Llama-2-7B-shaped stack, batch 8, budget 410) that is 32
wkv_step launches, one per layer, each doing append + attention + score update
+ select + merge for 256 (sequence, head) units.  Inputs are synthetic, seeded
and already resident in HBM when the timed region starts.  Prints ONE JSON line.

What the line carries:
  value / ms_per_step   median over --reps timed regions of --steps tokens each (min and max in
                        config.repetitions), wall clock around each region;
  roofline              algorithmic bytes per launch / average launch duration (HIP events around
                        the same regions) against the 8 TB/s HBM peak -- and against what a plain
                        streaming read with the same grid and byte count reaches in this run
                        (achievable_peak, frac_of_achievable), measured through wkv_probe_read; next to it
                        what the stack would take if its launches could overlap at their ends
                        (layers_unordered: two streams in turn; no valid order for layers that feed each
                        other, a yardstick for the cost of the launch boundaries);
  also                  the other configurations (cfg2, cfg4, cfg5), each with its own roofline;
                        cache_resident marks those whose whole K and V fit the 256 MB last-level
                        cache, whose fraction is therefore no HBM figure; for those, as_stack is the
                        same shape as a stack of handles stepped in turn (enough of them, up to 32,
                        that no row survives in the cache until its next use): the HBM figure;
  prefill               the bulk prefill of one layer, priced per contraction at its own MFMA peak;
  cpu_baseline          the CPU oracle on the host cores, all threads and one thread.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
LAST_LEVEL_CACHE = 256 << 20     # MI355X memory-side cache
FP64_MFMA_TFLOPS = 78.6          # MI355X published dense peaks
HALF_MFMA_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--reps", type=int, default=5, help="timed regions of --steps tokens each; the median is reported")
    ap.add_argument("--workload", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--layers", type=int, default=0, help="override the number of stacked layers")
    ap.add_argument("--threads", type=int, default=0, help="workgroup size override (256/512/1024)")
    ap.add_argument("--loads", choices=("auto", "cached", "streaming"), default="auto",
                    help="how cached rows are loaded (wkv_options.streaming); auto = the library decides")
    ap.add_argument("--split", type=int, default=0, help="workgroups per unit override (1/2/4/8/16; 0 = library's choice)")
    ap.add_argument("--prefill-tokens", type=int, default=4096,
                    help="prompt length of the bulk-prefill leg reported under 'prefill' (0 = skip it)")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--also", default="cfg2,cfg4,cfg5",
                    help="comma-separated workloads measured in the same run and reported under 'also' ('' = none)")
    ap.add_argument("--skip-probe", action="store_true", help="leave out the streaming-read yardstick")
    ap.add_argument("--skip-stacks", action="store_true",
                    help="leave out the stacked (HBM-resident) variant of the cache-resident side workloads")
    ap.add_argument("--cpu-core-seconds", type=float, default=30.0,
                    help="target CPU work (seconds x threads) of the oracle leg at all threads")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain device copy of known size (for scaling rocprofv3 byte counters)")
    return ap.parse_args()


def calibrate_copy():
    """A plain copy kernel of known size: 64 launches, each reading and writing 1 GiB.
    Under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE) the counter value per dispatch divided
    by 1 GiB is the factor by which the counter has to be scaled on this machine."""
    import torch
    n = 1 << 30
    src = torch.full((n,), 3, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(64):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibration": "device copy", "bytes_read_per_launch": n, "bytes_written_per_launch": n,
                      "launches": 64}))


def measured_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary has been committed."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    try:
        with open(path) as f:
            return json.load(f).get("hbm_bytes_per_launch")
    except (OSError, ValueError):
        return None


def main():
    args = parse()
    if args.calibrate_copy:
        calibrate_copy()
        return
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (units are independent and would shard "
              "with no exchange, but no multi-GPU path exists); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2503_01330_amd import binding as wkv
    from paper_2503_01330_amd import synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    W, K, REPS = args.warmup, args.steps, max(args.reps, 1)

    def run_workload(name, layers, threads, split=0):
        """Stage the stream, fill the cache, warm up, time REPS regions of K steps each."""
        cfg = synth.CONFIGS[name]
        layers = layers or cfg.layers
        fill = cfg.budget                       # tokens streamed (untimed) until the cache is full
        total = fill + W + (REPS + 1) * K     # (+1: the two-stream yardstick below)
        cfg = synth.scaled(cfg, steps=total, layers=max(layers, cfg.layers))
        code = synth.DTYPE_CODE[cfg.dtype]
        eb = synth.DTYPE_BYTES[cfg.dtype]
        # the whole synthetic stream resident in HBM, one [total, units, d] tensor triple per layer
        t0 = time.perf_counter()
        caches, bufs, ptrs = [], [], []
        for layer in range(layers):
            q, k, v = synth.Stream(cfg, layer).steps(0, total)
            tq, tk, tv = (torch.from_numpy(x).to(dev) for x in (q, k, v))
            out = torch.empty_like(tq)
            bufs.append((tq, tk, tv, out))
            ptrs.append(tuple(x.data_ptr() for x in (tq, tk, tv, out)))
            caches.append(wkv.Cache(cfg.batch, cfg.heads, cfg.head_dim, cfg.budget, cfg.recent, code,
                                    threads=threads, split=split,
                                    streaming={"auto": 0, "cached": 1, "streaming": 2}[args.loads]))
        gen_s = time.perf_counter() - t0
        stride = cfg.units * cfg.head_dim * eb
        stream = torch.cuda.current_stream().cuda_stream
        handles = [c.h for c in caches]
        step = wkv.wkv_step

        def run(t_lo, t_hi):
            for t in range(t_lo, t_hi):
                off = t * stride
                for h, (pq, pk, pv, po) in zip(handles, ptrs):
                    step(h, pq + off, pk + off, pv + off, po + off, stream)

        run(0, fill)                 # fill phase: cache grows to its budget
        run(fill, fill + W)          # steady-state warmup
        torch.cuda.synchronize()
        walls, evs = [], []
        for r in range(REPS):
            lo = fill + W + r * K
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            w0 = time.perf_counter()
            ev0.record()
            run(lo, lo + K)
            ev1.record()
            torch.cuda.synchronize()
            walls.append(time.perf_counter() - w0)
            evs.append(ev0.elapsed_time(ev1))
        # What the launch boundaries cost: the same steps once more, the handles of the stack taken from two
        # streams in turn, so that a launch starts on compute units as the one before leaves them.  No valid
        # order for a model (a layer's q, k, v follow from the layer before; here they are staged
        # inputs, and every handle keeps its own stream, so the results are the same): a yardstick only.
        unordered_us = None
        if layers >= 2 and layers % 2 == 0 and not args.skip_probe:
            side = torch.cuda.Stream()
            first = torch.cuda.current_stream()
            side.wait_stream(first)
            two = (first.cuda_stream, side.cuda_stream)
            lo = fill + W + REPS * K
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for t in range(lo, lo + K):
                off = t * stride
                for i, (h, (pq, pk, pv, po)) in enumerate(zip(handles, ptrs)):
                    step(h, pq + off, pk + off, pv + off, po + off, two[i & 1])
            first.wait_stream(side)
            ev1.record()
            torch.cuda.synchronize()
            unordered_us = ev0.elapsed_time(ev1) * 1e3 / (K * layers)
        step_bytes = caches[0].step_bytes()              # algorithmic bytes of one launch
        # which kernel the library launches for this shape: the sliced one allocates scratch
        o = caches[0].opt
        one = wkv.make_options(o.batch, o.heads, o.head_dim, o.budget, o.recent_window, o.dtype, split=1)
        kernel = "wkv_split_kernel" if wkv.wkv_workspace_bytes(o) > wkv.wkv_workspace_bytes(one) else "wkv_step_kernel"
        grid = wkv.wkv_launch_shape(o)
        for c in caches:
            c.close()
        del bufs
        torch.cuda.empty_cache()
        wall = statistics.median(walls)
        kernel_us = statistics.median(evs) * 1e3 / (K * layers)     # average launch duration incl. gaps (HIP events)
        kv_bytes = 2 * layers * cfg.units * (cfg.budget + 1) * cfg.head_dim * eb
        return dict(cfg=cfg, layers=layers, fill=fill, wall=wall, walls=walls, gen_s=gen_s, step_bytes=step_bytes,
                    kernel=kernel, kernel_us=kernel_us, achieved=step_bytes / (kernel_us * 1e-6) / 1e9,
                    tokens_per_s=cfg.batch * K / wall, grid=grid, kv_bytes=kv_bytes, unordered_us=unordered_us,
                    ev_us=[e * 1e3 / (K * layers) for e in evs])

    def probe(mm):
        """A plain streaming read with the launch shape and the byte count of one launch of mm, rotating
        over as many distinct slices of a buffer as the workload has layers (so that what is read comes
        from where the workload's rows come from: HBM for the 32-layer stack, the last-level cache for a
        single small handle).  Returns GB/s for cached and for non-temporal loads."""
        groups, threads = mm["grid"]
        quantum = 16 * groups
        nbytes = (mm["step_bytes"] + quantum - 1) // quantum * quantum
        slices = mm["layers"]
        buf = torch.empty(slices * nbytes, dtype=torch.uint8, device=dev)
        buf.fill_(1)
        stream = torch.cuda.current_stream().cuda_stream
        launches = max(K * mm["layers"], 64)
        res = {}
        for label, nt in (("cached", False), ("nontemporal", True)):
            times = []
            for r in range(REPS + 1):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(launches):
                    wkv.wkv_probe_read(buf.data_ptr() + (i % slices) * nbytes, nbytes, groups, threads, nt, 0, stream)
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            us = statistics.median(times[1:]) * 1e3 / launches
            res[label] = {"us_per_launch": round(us, 3), "GB/s": round(nbytes / (us * 1e-6) / 1e9, 1)}
        del buf
        torch.cuda.empty_cache()
        return res, nbytes

    def roofline(mm, workload):
        r = {"bound": "hbm", "achieved": round(mm["achieved"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
             "frac": round(mm["achieved"] / HBM_PEAK_GBS, 4), "traffic": measured_traffic(workload),
             "kernel": mm["kernel"], "bytes_per_launch": mm["step_bytes"],
             "avg_launch_us": round(mm["kernel_us"], 3),
             "avg_launch_us_min_max": [round(min(mm["ev_us"]), 3), round(max(mm["ev_us"]), 3)],
             "grid": {"workgroups": mm["grid"][0], "threads": mm["grid"][1]},
             "cache_resident": mm["kv_bytes"] <= LAST_LEVEL_CACHE}
        if not args.skip_probe:
            pr, nbytes = probe(mm)
            best = max(pr["cached"]["GB/s"], pr["nontemporal"]["GB/s"])
            r["achievable_peak"] = best
            r["frac_of_achievable"] = round(mm["achieved"] / best, 4)
            if mm["unordered_us"] is not None:
                r["layers_unordered"] = {"us_per_launch": round(mm["unordered_us"], 3),
                                         "frac": round(mm["step_bytes"] / (mm["unordered_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                         "what": "the same steps with the stack's handles taken from two streams in turn, "
                                                 "so that launches overlap at their ends; not a valid order for layers that "
                                                 "feed each other: what the launch boundaries cost"}
            r["streaming_read"] = {"bytes_per_launch": nbytes, **pr,
                                   "what": "wkv_probe_read: same grid, same bytes per launch, same number of rotating "
                                           "buffers as layers; reads only"}
        return r

    def describe(mm, workload):
        c = mm["cfg"]
        return (f"{workload}: {mm['layers']} layer(s) x batch {c.batch} x {c.heads} heads x {c.head_dim} {c.dtype}, "
                f"budget {c.budget}, recent window {c.recent}, steady state after a {mm['fill']}-token fill")

    m = run_workload(args.workload, args.layers, args.threads, args.split)
    cfg, layers, fill = m["cfg"], m["layers"], m["fill"]

    result = {
        "metric": "compressed-cache decode tokens/s at budget B; achieved HBM GB/s % of peak",
        "value": round(m["tokens_per_s"], 1), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(m["wall"] * 1e3 / K, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": {"fp16": "f16 in, f32/f64 accumulate", "bf16": "bf16 in, f32/f64 accumulate",
                                       "fp32": "f32 in, f64 accumulate"}[cfg.dtype],
        "data": "synthetic",
        "config": {"workload": describe(m, args.workload),
                   "units_per_launch": cfg.units, "launches_per_step": layers,
                   "threads_per_workgroup": args.threads or "auto",
                   "row_loads": args.loads,
                   "workgroups_per_unit": args.split or "auto",
                   "repetitions": {"timed_regions": REPS, "steps_each": K, "reported": "median",
                                   "ms_per_step_min_max": [round(min(m["walls"]) * 1e3 / K, 4),
                                                           round(max(m["walls"]) * 1e3 / K, 4)]},
                   "input_staging_s": round(m["gen_s"], 1)},
        "roofline": roofline(m, args.workload),
    }
    also = [w for w in args.also.split(",") if w and w != args.workload]
    if also:
        # the other configurations in the same run, reported next to the headline (not part of `value`)
        result["also"] = []
        for w in also:
            e = run_workload(w, 0, 0)
            entry = {"config": {"workload": describe(e, w)}, "value": round(e["tokens_per_s"], 1),
                     "unit": "tokens/s", "ms_per_step": round(e["wall"] * 1e3 / K, 4),
                     "roofline": roofline(e, w)}
            if entry["roofline"]["cache_resident"] and not args.skip_stacks:
                # One handle of this shape stays in the last-level cache from step to step, so the rate
                # above is not an HBM rate.  A model steps a stack of such handles in turn; with enough of
                # them (up to 32) that nothing survives until its next use, the same kernel reads from HBM.
                per_handle = e["kv_bytes"] // e["layers"]
                n = int(min(32, -(-2 * LAST_LEVEL_CACHE // per_handle)))
                st = run_workload(w, n, 0)
                entry["as_stack"] = {"config": {"workload": describe(st, w)}, "value": round(st["tokens_per_s"], 1),
                                     "unit": "tokens/s", "ms_per_step": round(st["wall"] * 1e3 / K, 4),
                                     "roofline": roofline(st, "-")}
            result["also"].append(entry)

    if args.prefill_tokens and cfg.dtype != "fp32" and cfg.head_dim <= 128:
        # bulk prefill of one layer's empty cache with a prompt (not part of `value`): the prompt rows attend
        # causally over the uncompressed prompt, then the cache is compressed to its budget
        P = min(args.prefill_tokens, wkv.WKV_MAX_PROMPT)
        pcfg = synth.scaled(cfg, steps=P)
        q, k, v = synth.Stream(pcfg, 0).steps(0, P)
        tq, tk, tv = (torch.from_numpy(x).to(dev) for x in (q, k, v))
        out = torch.empty_like(tq)
        code = synth.DTYPE_CODE[cfg.dtype]
        stream = torch.cuda.current_stream().cuda_stream
        times = []
        for rep_i in range(4):
            c = wkv.Cache(cfg.batch, cfg.heads, cfg.head_dim, cfg.budget, cfg.recent, code, max_prompt=P)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            wkv.wkv_prefill(c.h, tq.data_ptr(), tk.data_ptr(), tv.data_ptr(), out.data_ptr(), P, stream)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
            c.close()
        ms = statistics.median(times[1:])
        # The method's two contractions over the causal half, 2 flops per multiply-add: q.K^T (contracted in
        # fp64 here, for the score path's precision) and P.V (16-bit MFMA).  Algorithmic time = each once, at
        # its own dtype's peak.  What the kernels execute is more: q.K^T twice (rows, then column sums) and P.V
        # with the weights split into 2 (fp16) or 3 (bf16) 16-bit parts.
        half = 1.0 * cfg.units * P * (P + 1) * cfg.head_dim          # flops of one contraction
        algo_ms = (half / (FP64_MFMA_TFLOPS * 1e12) + half / (HALF_MFMA_TFLOPS * 1e12)) * 1e3
        parts = 2 if cfg.dtype == "fp16" else 3
        exec_ms = (2 * half / (FP64_MFMA_TFLOPS * 1e12) + parts * half / (HALF_MFMA_TFLOPS * 1e12)) * 1e3
        result["prefill"] = {
            "config": {"workload": f"{args.workload}: one layer, prompt of {P} tokens into an empty cache, "
                                   f"batch {cfg.batch} x {cfg.heads} heads x {cfg.head_dim} {cfg.dtype}, budget {cfg.budget}"},
            "value": round(cfg.batch * P / (ms * 1e-3), 1), "unit": "prompt tokens/s per layer", "ms": round(ms, 3),
            "roofline": {"bound": "mfma", "achieved": round(2 * half / (ms * 1e-3) / 1e12, 2), "peak": FP64_MFMA_TFLOPS,
                         "unit": "TFLOP/s", "frac": round(algo_ms / ms, 4), "traffic": None,
                         "kernel": "wkv_prefill_rows + wkv_prefill_scores + wkv_prefill_compress (one wkv_prefill call)",
                         "flops_per_contraction": half,
                         "algorithmic_ms": round(algo_ms, 3), "executed_flops_ms_at_peak": round(exec_ms, 3),
                         "frac_of_executed": round(exec_ms / ms, 4),
                         "note": "frac = algorithmic time / measured time, where algorithmic time prices q.K^T once at the "
                                 "fp64 MFMA peak (78.6 TFLOP/s) and P.V once at the 16-bit MFMA peak (2500 TFLOP/s); "
                                 "`achieved` is both contractions' flops over the whole call.  The kernels execute q.K^T "
                                 "twice (rows, then column sums: recomputed rather than stored) and P.V in 2-3 16-bit "
                                 "parts: frac_of_executed prices those flops instead"},
        }
        del tq, tk, tv, out
        torch.cuda.empty_cache()

    if not args.skip_cpu_baseline:
        import oracle
        # bounded sample: layer 0, every unit, steady-state steps after the same fill
        cores = oracle.threads()
        ocfg = synth.scaled(cfg, steps=fill + 4096 + 16)
        st = synth.Stream(ocfg, 0)
        orc = oracle.Oracle(cfg.units, cfg.head_dim, cfg.budget, cfg.recent, storage=cfg.dtype)
        q, k, v = (synth.storage_to_f32(x, cfg.dtype) for x in st.steps(0, fill))
        orc.run(q, k, v, want_out=False)
        probe_n = 16
        q, k, v = (synth.storage_to_f32(x, cfg.dtype) for x in st.steps(fill, fill + probe_n))
        c0 = time.perf_counter()
        orc.run(q, k, v)
        per = (time.perf_counter() - c0) / probe_n
        n = int(max(64, min(3072, args.cpu_core_seconds / (per * cores))))
        q, k, v = (synth.storage_to_f32(x, cfg.dtype) for x in st.steps(fill + probe_n, fill + probe_n + n))
        c0 = time.perf_counter()
        orc.run(q, k, v)
        cpu_s = time.perf_counter() - c0
        # the same oracle on one thread, a shorter slice of the same stream (about 10 s)
        n1 = int(max(8, min(1024, 10.0 / (per * cores))))
        lo = fill + probe_n + n
        q, k, v = (synth.storage_to_f32(x, cfg.dtype) for x in st.steps(lo, lo + n1))
        c0 = time.perf_counter()
        orc.run(q, k, v, threads=1)
        cpu1_s = time.perf_counter() - c0
        result["cpu_baseline"] = {
            "value": round(cfg.batch * n / (cpu_s * layers), 2), "unit": "tokens/s",
            "cores": cores, "kind": "oracle",
            "sample": f"layer 0 of {layers}, all {cfg.units} units, {n} steady-state steps in {cpu_s:.2f} s wall on "
                      f"{cores} threads after the {fill}-token fill; scaled by 1/{layers} layers to whole-token rate",
            "one_thread": {"value": round(cfg.batch * n1 / (cpu1_s * layers), 2), "unit": "tokens/s", "cores": 1,
                           "sample": f"the next {n1} steps of the same stream in {cpu1_s:.2f} s on one thread, scaled alike"},
        }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
