#!/usr/bin/env python3
"""Benchmark of the RMSNorm forward hot path on one MI355X (and, with --op, of the softmax,
LayerNorm, cross-entropy and row-sum kernels at the paper's own shapes, same protocol).

A step is one rmsnorm_fwd call over the headline workload (bf16, M = 16384,
N = 8192, eps = 1e-5; synthetic N(0,1) inputs, N(1,0.1) weight), with inputs
resident in HBM before the timed region.  The metric is achieved HBM GB/s by the
bytes model of the paper's kernel performance table (read x once, write y once,
plus the weight) and its fraction of the 8 TB/s peak.

Protocol: a settling phase of back-to-back launches (the first ~20 ms of work
after idle run in a clock transient in which kernels take up to 40 % longer; the
JSON line records how many launches it took as settle_launches), W warm-up
launches, then two measurements of K launches each.
  1. One timed region: K launches back to back, bracketed by device
     synchronisation and by a pair of events on the launch stream.  This is what
     `value`, `ms_per_step` and `roofline.achieved` / `roofline.frac` are computed
     from (`config.timing` says "back_to_back_region"): launches on one stream run
     with no gap between them, and the rocprofv3 kernel trace of the same command
     gives the same average duration per dispatch.
  2. The paper's Section 7 protocol: every launch inside its own event pair, the
     10 % trimmed mean of the K durations (also median and minimum).  An event
     pair around a single launch reads 1 to 2 us longer than the dispatch itself,
     so this figure is lower; it is reported next to the first one as
     `roofline.event_pair_trimmed_mean_us` and `roofline.frac_event_pair`.
Launches rotate over several buffer sets whose total size exceeds the 256 MB
Infinity Cache, so the figure is an HBM figure.  `roofline.traffic` is the HBM
bytes per launch that the hardware counters read in the committed rocprofv3 run
named by `roofline.traffic_source` (it is not re-measured by this script);
`roofline.traffic_gbps` is that traffic over this run's time per launch.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0
TRAFFIC_FILES = {
    "rmsnorm": "hbm_traffic_rmsnorm_bf16_16384x8192.txt",
    "softmax": "hbm_traffic_softmax_fp16_8192x8192.txt",
    "softmax_attention": "hbm_traffic_softmax_fp16_170320x197.txt",   # --attention-len 197
    "layernorm": "hbm_traffic_layernorm_fp16_8192x4096.txt",
    "crossentropy": "hbm_traffic_crossentropy_fp16_8192x32000.txt",
    "rowsum": "hbm_traffic_rowsum_fp16_8192x8192.txt",
}


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def read_traffic(op: str = "rmsnorm"):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of `op`, or None."""
    try:
        text = open(os.path.join(ROOT, "profiles", TRAFFIC_FILES[op])).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, flags=re.M)
    return float(m.group(1)) if m else None


def trimmed_mean(values, frac=0.10):
    v = sorted(values)
    cut = int(len(v) * frac)
    core = v[cut:len(v) - cut] if len(v) > 2 * cut else v
    return sum(core) / len(core)


def settle(launchers, ms: float) -> int:
    """Untimed back-to-back launches for about `ms` milliseconds of GPU time: lets the clocks
    settle after idle before anything is measured.  Returns how many launches that took."""
    import torch
    if ms <= 0:
        return 0
    n = len(launchers)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    done, spent = 0, 0.0
    while spent < ms and done < 200000:
        a.record()
        for i in range(100):
            launchers[(done + i) % n]()
        b.record()
        torch.cuda.synchronize()
        spent += a.elapsed_time(b)
        done += 100
    log(f"settled: {done} launches, {spent:.1f} ms")
    return done


def timed_region(launchers, K: int):
    """K back-to-back launches inside one event pair; returns milliseconds per step."""
    import torch
    n = len(launchers)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(K):
        launchers[i % n]()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / K


def per_launch_us(launchers, K: int):
    """K launches, each inside its own event pair; returns the durations in microseconds."""
    import torch
    n = len(launchers)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
             for _ in range(K)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(pairs):
        a.record()
        launchers[i % n]()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) * 1e3 for a, b in pairs]


def copy_ceiling(srcs, dsts, K: int, W: int, staged: bool = False) -> dict:
    """The measurement library's streaming copy over the same buffers with the same protocol
    (W warm-up launches, K back to back in one event pair): what a stream that is half reads
    and half writes reaches at this launch size, launch and ramp-up included.  With `staged`
    also the copy that goes through LDS tiles in workgroups of 256 threads, the ceiling of the
    kernels that stage short rows that way."""
    from paper_2603_21331_amd import measure
    import torch
    n = len(srcs)
    # the copies move whole 16-byte vectors: at most 15 bytes of a buffer are left out
    whole = srcs[0].numel() * srcs[0].element_size() // 16 * 16
    srcs = [t.view(-1).view(torch.uint8)[:whole] for t in srcs]
    dsts = [t.view(-1).view(torch.uint8)[:whole] for t in dsts]
    nbytes = 2 * whole
    out = {}
    entries = [("copy", measure.measure_copy)] + ([("staged_copy", measure.measure_staged_copy)] if staged else [])
    for name, entry in entries:
        copies = [(lambda i=i: entry(srcs[i], dsts[i])) for i in range(n)]
        for i in range(W):
            copies[i % n]()
        us = timed_region(copies, K) * 1e3
        out[f"{name}_mean_us"] = round(us, 3)
        out[f"{name}_ceiling_gbps"] = round(nbytes / (us * 1e-6) / 1e9, 1)
    return out


def roofline_object(nbytes: int, ms_per_step: float, durs_us, traffic=None, traffic_source=None,
                    **extra):
    """The roofline object of the JSON line.  achieved / frac: algorithmic bytes over the time
    per launch of the back-to-back region; frac_event_pair: the same bytes over the 10 %
    trimmed mean of the per-launch event pairs; traffic: counter-derived HBM bytes per launch
    from the committed profile `traffic_source`, traffic_gbps: those bytes over this run's time
    per launch."""
    achieved = nbytes / (ms_per_step * 1e-3) / 1e9
    pair_us = trimmed_mean(durs_us)
    obj = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
           "frac": round(achieved / PEAK_HBM_GBPS, 4), "traffic": traffic,
           "traffic_source": traffic_source if traffic is not None else None,
           "traffic_gbps": round(traffic / (ms_per_step * 1e-3) / 1e9, 1) if traffic else None,
           "region_us_per_launch": round(ms_per_step * 1e3, 3),
           "event_pair_trimmed_mean_us": round(pair_us, 3),
           "frac_event_pair": round(nbytes / (pair_us * 1e-6) / 1e9 / PEAK_HBM_GBPS, 4),
           "event_pair_median_us": round(sorted(durs_us)[len(durs_us) // 2], 3),
           "event_pair_min_us": round(min(durs_us), 3)}
    obj.update(extra)
    return obj


def traffic_fields(op: str) -> dict:
    """traffic and traffic_source arguments of roofline_object for `op`."""
    return {"traffic": read_traffic(op), "traffic_source": "profiles/" + TRAFFIC_FILES[op]}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--buffer-sets", type=int, default=4,
                    help="x/y buffer pairs cycled through (4 x 512 MiB defeats the Infinity Cache)")
    ap.add_argument("--threads-per-row", type=int, default=0,
                    help="force the block size through rmsnorm_fwd_tuned (0 = automatic dispatch)")
    ap.add_argument("--rows", type=int, default=16384, help="M (the headline workload is 16384)")
    ap.add_argument("--cols", type=int, default=8192,
                    help="N (the headline workload is 8192; other values run the same bf16 recipe at "
                         "that row length, e.g. 197 for rows that are not 16-byte aligned)")
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed back-to-back launches for this many milliseconds before the "
                         "warm-up, so that the clock transient after idle is over (0 = none; "
                         "measured with a timed region of 20 launches: 20 ms of settling leave the "
                         "figure 1 to 1.5 %% low, 60 and 200 ms give the same)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all-configs", action="store_true",
                    help="after the headline measurement, also time the other four workloads "
                         "(GPU and oracle) and add them to the JSON line under other_configs")
    ap.add_argument("--op", choices=["rmsnorm", "softmax", "layernorm", "crossentropy", "rowsum"],
                    default="rmsnorm",
                    help="rmsnorm (default): the headline benchmark.  softmax / layernorm / "
                         "crossentropy / rowsum: the same protocol on the next kernels at the paper's "
                         "largest shape for each (fp16 8192 x 8192; fp16 8192 x 4096; fp16 "
                         "8192 x 32000; fp16 8192 x 8192)")
    ap.add_argument("--paper-shape", type=int, choices=[0, 1], default=None,
                    help="with --op: which of the kernel's two FP16 rows of the paper's performance "
                         "table to run.  softmax: 0 = 4096 x 4096, 1 = 8192 x 8192 (default); "
                         "layernorm: 0 = 4096 x 5120, 1 = 8192 x 4096 (default); crossentropy: "
                         "0 = 4096 x 32000, 1 = 8192 x 32000 (default); rowsum: 0 = 8192 x 8192 "
                         "(default), 1 = 16384 x 4096.  The committed traffic summaries are those of "
                         "the default shapes; for the other shape `traffic` is null")
    ap.add_argument("--attention-len", type=int, default=0,
                    help="with --op softmax or layernorm: instead of the paper's shape, 64 MiB of "
                         "fp16 rows of this many elements (e.g. the 197 positions of an attention "
                         "row: not 16-byte aligned, several rows per workgroup through LDS)")
    ap.add_argument("--shape", type=int, nargs=2, metavar=("M", "N"), default=None,
                    help="with --op layernorm: fp16 M x N of the same recipe instead of the paper's "
                         "shape (e.g. 32768 5120, a launch large enough for the work-queue form of "
                         "the resident kernel); `traffic` is null")
    ap.add_argument("--profile-only", action="store_true",
                    help="warm-up plus --steps launches and nothing else (for rocprofv3 runs)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="with --profile-only: also launch the library's streaming copy on the "
                         "same buffers (known traffic, for scaling the hardware counters)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this benchmark is single-GPU by construction (rows are independent; "
              "more GPUs would only shard M); run it with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2603_21331_amd import binding, inputs, measure

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    if not os.path.exists(binding.library_path()):
        print("bench.py: librmsnorm_hip.so is not built (run __graft_entry__.build())", file=sys.stderr)
        return 2
    binding.load()
    measure.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.op == "softmax":
        return bench_softmax(args, dev)
    if args.op == "layernorm":
        return bench_layernorm(args, dev)
    if args.op == "crossentropy":
        return bench_crossentropy(args, dev)
    if args.op == "rowsum":
        return bench_rowsum(args, dev)

    M, K, W, S = args.rows, args.steps, args.warmup, max(1, args.buffer_sets)
    t0 = time.time()
    if args.cols == 8192:
        case = inputs.config3(M=M)
    else:                                       # the same recipe (streams 48 / 49) at another row length
        case = inputs.random_case(0, 48, M, args.cols, inputs.BF16, 1e-5)
    N, eps, dtype = case["N"], case["eps"], case["dtype"]
    log(f"generated {case['name']} in {time.time() - t0:.1f} s")
    nbytes = inputs.algorithmic_bytes(M, N, dtype)

    x_host = torch.from_numpy(case["x"].view(np.int16))
    w_dev = torch.from_numpy(case["w"].view(np.int16)).to(dev).view(torch.bfloat16)
    xs, ys = [], []
    if args.cols != 8192 and 2 * M * N * 2 < (256 << 20):
        S = max(S, min(32, (1 << 30) // (2 * M * N * 2)))       # at least 1 GiB of buffers in rotation
    for _ in range(S):
        xs.append(x_host.to(dev).view(torch.bfloat16))
        ys.append(torch.empty((M, N), dtype=torch.bfloat16, device=dev))
    auto_threads = binding.rmsnorm_auto_threads_per_row(N, dtype)
    variant = binding.VARIANT_NAMES[binding.rmsnorm_select_variant(xs[0], w_dev, ys[0])]
    plan = None
    if variant == "queue" and not args.threads_per_row:
        _, grid, shards, block_rows, prefetch = binding.rmsnorm_queue_plan(M, N, dtype)
        plan = {"resident_workgroups": grid, "threads_per_workgroup": 512, "shards": shards,
                "rows_per_block": block_rows, "prefetch": prefetch}
    launchers = [binding.bind_rmsnorm_fwd(xs[i], w_dev, ys[i], eps,
                                          threads_per_row=args.threads_per_row) for i in range(S)]
    torch.cuda.synchronize()

    settled = settle(launchers, args.settle_ms)
    for i in range(W):
        launchers[i % S]()
    torch.cuda.synchronize()

    if args.profile_only:
        for i in range(K):
            launchers[i % S]()
        if args.calib_copy:
            for i in range(K):
                measure.measure_copy(xs[i % S], ys[i % S])
        torch.cuda.synchronize()
        log("profile-only run done")
        return 0

    # ---- timed region: K steps, whole-job throughput and the kernel's average duration ----
    wall0 = time.perf_counter()
    ms_per_step = timed_region(launchers, K)
    wall = time.perf_counter() - wall0
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    log(f"region: {K} steps, {ms_per_step * 1e3:.2f} us per step (wall {wall * 1e3:.1f} ms) "
        f"-> {value:.0f} GB/s")

    # ---- per-launch durations (the paper's protocol: one event pair per launch) -----------
    durs_us = per_launch_us(launchers, K)
    log(f"event pairs: trimmed {trimmed_mean(durs_us):.2f} us, "
        f"median {sorted(durs_us)[len(durs_us) // 2]:.2f} us, min {min(durs_us):.2f} us")

    # same-buffer figure (cache-assisted; reported for contrast only)
    pairs1 = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(min(K, 50))]
    for a, b in pairs1:
        a.record()
        launchers[0]()
        b.record()
    torch.cuda.synchronize()
    same_us = trimmed_mean([a.elapsed_time(b) * 1e3 for a, b in pairs1])

    # streaming-copy ceiling on the same buffers (2 * M * N * 2 bytes, no weight), same protocol
    ceiling = copy_ceiling(xs, ys, K, W, staged=N * 2 < 2048)

    result = {
        "metric": f"RMSNorm fwd achieved HBM GB/s and % of MI355X peak (bf16, {M}x{N})",
        "value": round(value, 1),
        "unit": "GB/s",
        "pct_of_peak": round(100.0 * value / PEAK_HBM_GBPS, 2),
        "rows_per_s": round(M / (ms_per_step * 1e-3), 1),
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "settle_launches": settled,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"rmsnorm_fwd bf16 M={M} N={N} eps={eps}" +
                        (" (configs[2], headline shape)" if (M, N) == (16384, 8192) else ""),
            "storage_dtype": "bf16",
            "timing": "back_to_back_region",
            "threads_per_row": args.threads_per_row or (512 if plan else auto_threads),
            "dispatch": "forced" if args.threads_per_row else "auto",
            "kernel": "block" if args.threads_per_row else variant,
            "queue_plan": plan,
            "buffer_sets": S,
            "bytes_per_step": nbytes,
        },
        "roofline": roofline_object(nbytes, ms_per_step, durs_us,
                                    **(traffic_fields("rmsnorm") if (M, N) == (16384, 8192) else {}),
                                    same_buffer_trimmed_mean_us=round(same_us, 3), **ceiling),
    }

    # ---- CPU baseline: the oracle as it stands, on the host cores -------------------------
    if not args.no_cpu_baseline:
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import compare
        cores = oracle.hardware_threads()
        best = None
        y_ref = None
        for _ in range(3):
            t = time.perf_counter()
            y_ref = oracle.rmsnorm_oracle(case["x"], case["w"], eps, dtype, nthreads=cores)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
        t = time.perf_counter()
        rows1 = min(M, 1024)
        oracle.rmsnorm_oracle(case["x"][:rows1], case["w"], eps, dtype, nthreads=1)
        dt1 = time.perf_counter() - t
        result["cpu_baseline"] = {
            "value": round(nbytes / best / 1e9, 3),
            "unit": "GB/s",
            "cores": cores,
            "kind": "oracle",
            "sample": f"the whole workload ({M} x {N}), best of 3 runs, {best:.3f} s each",
            "rows_per_s": round(M / best, 1),
            "single_thread_gbps": round(inputs.algorithmic_bytes(rows1, N, dtype) / dt1 / 1e9, 3),
            "single_thread_sample": f"first {rows1} rows, one run",
        }
        log(f"oracle: {best:.3f} s on {cores} threads")
        launchers[0]()          # the copy-ceiling pass overwrote the outputs
        torch.cuda.synchronize()
        got = ys[0].view(torch.int16).cpu().numpy().view(np.uint16)
        stats = compare.check_parity(got, y_ref, dtype, "bench output vs oracle")
        result["parity"] = {"checked": "every element of one output buffer", **stats}

    if args.all_configs:
        del xs, ys, launchers
        torch.cuda.empty_cache()
        result["other_configs"] = other_configs(dev, K)

    print(json.dumps(result), flush=True)
    return 0


def bench_softmax(args, dev) -> int:
    """Row softmax, fp16, 8192 x 8192 (the largest softmax row of the paper's performance
    table: 95.9 us, 2800 GB/s on H100), same protocol as the headline benchmark."""
    import numpy as np
    import torch
    from paper_2603_21331_amd import inputs, measure, softmax

    softmax.load()
    measure.load()
    n, K, W, S = (4096 if args.paper_shape == 0 else 8192), args.steps, args.warmup, max(1, args.buffer_sets)
    if n == 4096:
        S = max(S, 8)                          # 8 x 64 MiB: past the Infinity Cache
    t0 = time.time()
    if args.attention_len:
        # attention scores over a context of `cols` positions (odd lengths such as 77, 197, 257:
        # the rows are not 16-byte aligned and take the LDS-staged kernel); 64 MiB of them
        cols = args.attention_len
        n = (64 << 20) // (2 * cols) // 8 * 8      # whole 16-byte vectors in total, for the calibration copy
        S = max(S, 8)
        case = inputs.softmax_case(0, 100, n, cols, inputs.FP16, 2.0)
    else:
        cols = n
        case = inputs.softmax_paper_shape(n)
    log(f"generated {case['name']} in {time.time() - t0:.1f} s")
    nbytes = inputs.softmax_bytes(n, cols, inputs.FP16)
    x_host = torch.from_numpy(case["x"].view(np.int16))
    xs = [x_host.to(dev).view(torch.float16) for _ in range(S)]
    ys = [torch.empty((n, cols), dtype=torch.float16, device=dev) for _ in range(S)]
    fns = [softmax.bind_softmax_fwd(xs[i], ys[i], threads_per_row=args.threads_per_row)
           for i in range(S)]
    settled = settle(fns, args.settle_ms)
    for i in range(W):
        fns[i % S]()
    torch.cuda.synchronize()
    if args.profile_only:
        for i in range(K):
            fns[i % S]()
        if args.calib_copy:
            for i in range(K):
                measure.measure_copy(xs[i % S], ys[i % S])
        torch.cuda.synchronize()
        log("profile-only run done")
        return 0
    ms_per_step = timed_region(fns, K)
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    durs = per_launch_us(fns, K)
    traffic = {}                               # summaries exist for 8192 x 8192 and for 197 positions
    if args.attention_len == 197:
        traffic = traffic_fields("softmax_attention")
    elif not args.attention_len and args.paper_shape != 0:
        traffic = traffic_fields("softmax")
    result = {
        "metric": f"Softmax fwd achieved HBM GB/s and % of MI355X peak (fp16, {n}x{cols})",
        "value": round(value, 1), "unit": "GB/s",
        "pct_of_peak": round(100.0 * value / PEAK_HBM_GBPS, 2),
        "rows_per_s": round(n / (ms_per_step * 1e-3), 1),
        "n_gpus": 1, "steps": K, "warmup": W, "settle_launches": settled,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"softmax_fwd fp16 M={n} N={cols}", "storage_dtype": "fp16",
                   "timing": "back_to_back_region",
                   "threads_per_row": args.threads_per_row
                   or softmax.softmax_auto_threads_per_row(cols, inputs.FP16),
                   "buffer_sets": S, "bytes_per_step": nbytes},
        "roofline": roofline_object(nbytes, ms_per_step, durs, **traffic),
    }
    y_keep = ys[0].clone()
    result["roofline"].update(copy_ceiling(xs, ys, K, W, staged=bool(args.attention_len)))
    ys[0].copy_(y_keep)
    if not args.no_cpu_baseline:
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import compare
        cores = oracle.hardware_threads()
        best, y_ref = None, None
        for _ in range(3):
            t = time.perf_counter()
            y_ref = oracle.softmax_oracle(case["x"], inputs.FP16, nthreads=cores)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
        result["cpu_baseline"] = {"value": round(nbytes / best / 1e9, 3), "unit": "GB/s",
                                  "cores": cores, "kind": "oracle",
                                  "sample": f"the whole workload ({n} x {cols}), best of 3 runs, "
                                            f"{best:.3f} s each"}
        got = ys[0].view(torch.int16).cpu().numpy().view(np.uint16)
        result["parity"] = {"checked": "every element of one output buffer",
                            **compare.check_softmax_parity(got, y_ref, inputs.FP16, "bench softmax")}
    print(json.dumps(result), flush=True)
    return 0


def bench_layernorm(args, dev) -> int:
    """LayerNorm forward, fp16, 8192 x 4096 (the larger LayerNorm row of the paper's performance
    table: 51.9 us, 2586 GB/s on H100), same protocol as the headline benchmark."""
    import numpy as np
    import torch
    from paper_2603_21331_amd import inputs, layernorm, measure

    layernorm.load()
    measure.load()
    K, W = args.steps, args.warmup
    which = 1 if args.paper_shape is None else args.paper_shape
    if args.attention_len:
        # 64 MiB of short rows (e.g. 197 elements: not 16-byte aligned, several per workgroup
        # through LDS), a whole number of 16-byte vectors in total for the copy beside it
        which = -1
        cols = args.attention_len
        case = inputs.layernorm_case(0, 130, (64 << 20) // (2 * cols) // 8 * 8, cols, inputs.FP16)
    elif args.shape:
        which = -1
        case = inputs.layernorm_case(0, 134, args.shape[0], args.shape[1], inputs.FP16)
    else:
        case = inputs.layernorm_paper_shape(which)
    M, N, eps = case["M"], case["N"], case["eps"]
    nbytes = inputs.layernorm_bytes(M, N, inputs.FP16)

    def queue_takes(m, n):
        try:
            return layernorm.layernorm_queue_plan(m, n, layernorm.LAYERNORM_DTYPE_FP16)[0]
        except layernorm.LayerNormError:
            return False

    S = max(args.buffer_sets, 8)               # 8 x 128 MiB: well past the Infinity Cache
    while S > 2 and S * 2 * M * N * 2 > (8 << 30):
        S -= 1                                 # (larger shapes: at most 8 GiB of buffers)
    as_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.float16)
    x0, wd, bd = as_dev(case["x"]), as_dev(case["w"]), as_dev(case["b"])
    xs = [x0] + [x0.clone() for _ in range(S - 1)]
    ys = [torch.empty_like(x0) for _ in range(S)]
    fns = [layernorm.bind_layernorm_fwd(xs[i], wd, bd, ys[i], eps,
                                        threads_per_row=args.threads_per_row) for i in range(S)]
    settled = settle(fns, args.settle_ms)
    for i in range(W):
        fns[i % S]()
    torch.cuda.synchronize()
    if args.profile_only:
        for i in range(K):
            fns[i % S]()
        if args.calib_copy:
            for i in range(K):
                measure.measure_copy(xs[i % S], ys[i % S])
        torch.cuda.synchronize()
        log("profile-only run done")
        return 0
    ms_per_step = timed_region(fns, K)
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    durs = per_launch_us(fns, K)
    result = {
        "metric": f"LayerNorm fwd achieved HBM GB/s and % of MI355X peak (fp16, {M}x{N})",
        "value": round(value, 1), "unit": "GB/s",
        "pct_of_peak": round(100.0 * value / PEAK_HBM_GBPS, 2),
        "rows_per_s": round(M / (ms_per_step * 1e-3), 1),
        "n_gpus": 1, "steps": K, "warmup": W, "settle_launches": settled,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"layernorm_fwd fp16 M={M} N={N} eps={eps} with bias",
                   "storage_dtype": "fp16", "timing": "back_to_back_region",
                   "threads_per_row": args.threads_per_row
                   or layernorm.layernorm_auto_threads_per_row(N, inputs.FP16),
                   "work_queue": bool(not args.threads_per_row and queue_takes(M, N)),
                   "buffer_sets": S, "bytes_per_step": nbytes},
        "roofline": roofline_object(nbytes, ms_per_step, durs,
                                    **(traffic_fields("layernorm") if which == 1 else {})),
    }
    y_keep = ys[0].clone()
    result["roofline"].update(copy_ceiling(xs, ys, K, W, staged=bool(args.attention_len)))
    ys[0].copy_(y_keep)
    if not args.no_cpu_baseline:
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import compare
        cores = oracle.hardware_threads()
        best = None
        for _ in range(3):
            t = time.perf_counter()
            y_ref, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], eps,
                                                        inputs.FP16, nthreads=cores, stats=True)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
        result["cpu_baseline"] = {"value": round(nbytes / best / 1e9, 3), "unit": "GB/s",
                                  "cores": cores, "kind": "oracle",
                                  "sample": f"the whole workload ({M} x {N}), best of 3 runs, "
                                            f"{best:.3f} s each"}
        f64 = lambda a: inputs.storage_to_f64(a, inputs.FP16)
        scale = compare.layernorm_scale(f64(case["x"]), f64(case["w"]), f64(case["b"]), mean, rstd)
        got = ys[0].view(torch.int16).cpu().numpy().view(np.uint16)
        result["parity"] = {"checked": "every element of one output buffer",
                            **compare.check_layernorm_parity(got, y_ref, scale, inputs.FP16,
                                                             "bench layernorm")}
    print(json.dumps(result), flush=True)
    return 0


def bench_crossentropy(args, dev) -> int:
    """Cross-entropy forward, fp16, 8192 x 32000 (the larger cross_ent row of the paper's
    performance table: 253.3 us, 2070 GB/s on H100), same protocol as the headline benchmark."""
    import numpy as np
    import torch
    from paper_2603_21331_amd import crossentropy, inputs, measure

    crossentropy.load()
    measure.load()
    K, W, S = args.steps, args.warmup, max(1, args.buffer_sets)
    t0 = time.time()
    which = 1 if args.paper_shape is None else args.paper_shape
    case = inputs.crossentropy_paper_shape(which)
    M, N = case["M"], case["N"]
    log(f"generated {case['name']} in {time.time() - t0:.1f} s")
    nbytes = inputs.crossentropy_bytes(M, N, inputs.FP16)
    x0 = torch.from_numpy(case["x"].view(np.int16)).to(dev).view(torch.float16)
    td = torch.from_numpy(case["target"]).to(dev)
    xs = [x0] + [x0.clone() for _ in range(S - 1)]          # 4 x 500 MiB: past the Infinity Cache
    losses = [torch.empty(M, dtype=torch.float32, device=dev) for _ in range(S)]
    fns = [crossentropy.bind_crossentropy_fwd(xs[i], td, losses[i], None,
                                              threads_per_row=args.threads_per_row) for i in range(S)]
    settled = settle(fns, args.settle_ms)
    for i in range(W):
        fns[i % S]()
    torch.cuda.synchronize()
    if args.profile_only:
        for i in range(K):
            fns[i % S]()
        if args.calib_copy:             # every buffer set holds the same logits: copying one
            for i in range(K):          # onto the next changes nothing
                measure.measure_copy(xs[i % S], xs[(i + 1) % S])
        torch.cuda.synchronize()
        log("profile-only run done")
        return 0
    ms_per_step = timed_region(fns, K)
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    durs = per_launch_us(fns, K)
    result = {
        "metric": f"Cross-entropy fwd achieved HBM GB/s and % of MI355X peak (fp16, {M}x{N})",
        "value": round(value, 1), "unit": "GB/s",
        "pct_of_peak": round(100.0 * value / PEAK_HBM_GBPS, 2),
        "rows_per_s": round(M / (ms_per_step * 1e-3), 1),
        "n_gpus": 1, "steps": K, "warmup": W, "settle_launches": settled,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"crossentropy_fwd fp16 M={M} N={N}, int64 targets, fp32 loss per row",
                   "storage_dtype": "fp16", "timing": "back_to_back_region",
                   "threads_per_row": args.threads_per_row
                   or crossentropy.crossentropy_auto_threads_per_row(N, inputs.FP16),
                   "buffer_sets": S, "bytes_per_step": nbytes},
        "roofline": roofline_object(nbytes, ms_per_step, durs,
                                    **(traffic_fields("crossentropy") if which == 1 else {})),
    }
    if not args.no_cpu_baseline:
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import compare
        cores = oracle.hardware_threads()
        best, ref = None, None
        for _ in range(2):
            t = time.perf_counter()
            ref = oracle.crossentropy_oracle(case["x"], case["target"], inputs.FP16, nthreads=cores)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
        result["cpu_baseline"] = {"value": round(nbytes / best / 1e9, 3), "unit": "GB/s",
                                  "cores": cores, "kind": "oracle",
                                  "sample": f"the whole workload ({M} x {N}), best of 2 runs, "
                                            f"{best:.3f} s each"}
        got = losses[0].cpu().numpy()
        result["parity"] = {"checked": "every loss of one output buffer",
                            **compare.check_crossentropy_parity(got, ref, "bench crossentropy")}
    print(json.dumps(result), flush=True)
    return 0


def bench_rowsum(args, dev) -> int:
    """Row sum, fp16, 8192 x 8192 (the first reduce row of the paper's performance table:
    62.2 us, 2156 GB/s on H100; --paper-shape 1 selects its second row, 16384 x 4096), same
    protocol as the headline benchmark."""
    import numpy as np
    import torch
    from paper_2603_21331_amd import inputs, measure, rowsum

    rowsum.load()
    measure.load()
    K, W = args.steps, args.warmup
    which = 0 if args.paper_shape is None else args.paper_shape
    case = inputs.rowsum_paper_shape(which)
    M, N = case["M"], case["N"]
    nbytes = inputs.rowsum_bytes(M, N, inputs.FP16)
    S = max(args.buffer_sets, 8)               # 8 x 128 MiB: well past the Infinity Cache
    x0 = torch.from_numpy(case["x"].view(np.int16)).to(dev).view(torch.float16)
    xs = [x0] + [x0.clone() for _ in range(S - 1)]
    ys = [torch.empty(M, dtype=torch.float32, device=dev) for _ in range(S)]
    fns = [rowsum.bind_rowsum_fwd(xs[i], ys[i], threads_per_row=args.threads_per_row)
           for i in range(S)]
    settled = settle(fns, args.settle_ms)
    for i in range(W):
        fns[i % S]()
    torch.cuda.synchronize()
    if args.profile_only:
        for i in range(K):
            fns[i % S]()
        if args.calib_copy:             # every buffer set holds the same values: copying one
            for i in range(K):          # onto the next changes nothing
                measure.measure_copy(xs[i % S], xs[(i + 1) % S])
        torch.cuda.synchronize()
        log("profile-only run done")
        return 0
    ms_per_step = timed_region(fns, K)
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    durs = per_launch_us(fns, K)
    result = {
        "metric": f"Row-sum reduce achieved HBM GB/s and % of MI355X peak (fp16, {M}x{N})",
        "value": round(value, 1), "unit": "GB/s",
        "pct_of_peak": round(100.0 * value / PEAK_HBM_GBPS, 2),
        "rows_per_s": round(M / (ms_per_step * 1e-3), 1),
        "n_gpus": 1, "steps": K, "warmup": W, "settle_launches": settled,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"rowsum_fwd fp16 M={M} N={N}, fp32 sum per row",
                   "storage_dtype": "fp16", "timing": "back_to_back_region",
                   "threads_per_row": args.threads_per_row
                   or rowsum.rowsum_auto_threads_per_row(N, inputs.FP16),
                   "buffer_sets": S, "bytes_per_step": nbytes},
        "roofline": roofline_object(nbytes, ms_per_step, durs,
                                    **(traffic_fields("rowsum") if which == 0 else {})),
    }
    if not args.no_cpu_baseline:
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import compare
        cores = oracle.hardware_threads()
        best, ref = None, None
        for _ in range(3):
            t = time.perf_counter()
            ref = oracle.rowsum_oracle(case["x"], inputs.FP16, nthreads=cores, with_abs=True)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
        result["cpu_baseline"] = {"value": round(nbytes / best / 1e9, 3), "unit": "GB/s",
                                  "cores": cores, "kind": "oracle",
                                  "sample": f"the whole workload ({M} x {N}), best of 3 runs, "
                                            f"{best:.3f} s each"}
        got = ys[0].cpu().numpy()
        result["parity"] = {"checked": "every sum of one output buffer",
                            **compare.check_rowsum_parity(got, ref[0], ref[1], N, "bench rowsum")}
    print(json.dumps(result), flush=True)
    return 0


def other_configs(dev, iters: int):
    """GPU time (rotating buffers; per-launch events, 10 % trimmed mean, and back-to-back
    launches inside one event pair) and oracle time (single thread and all threads, best of 3)
    for the workloads other than the headline: the other four configurations and the three
    FP16 shapes of the paper's own RMSNorm rows (39.1, 51.2 and 96.3 us on H100)."""
    import numpy as np
    import torch
    import oracle
    from paper_2603_21331_amd import binding, inputs

    cases = [inputs.config1(), inputs.config2()] + [inputs.config4(n) for n in inputs.CONFIG4_N] \
        + [inputs.config5()] + [inputs.rmsnorm_paper_shape(k) for k in range(3)]
    tdt = {inputs.FP32: torch.float32, inputs.FP16: torch.float16, inputs.BF16: torch.bfloat16}
    cores = oracle.hardware_threads()
    out = []
    for case in cases:
        M, N, dtype, eps = case["M"], case["N"], case["dtype"], case["eps"]
        nbytes = inputs.algorithmic_bytes(M, N, dtype)
        sets = max(2, min(8, (1 << 30) // max(nbytes, 1) + 1))
        if dtype == inputs.FP32:
            x0 = torch.from_numpy(case["x"]).to(dev)
            w = torch.from_numpy(case["w"]).to(dev)
        else:
            x0 = torch.from_numpy(case["x"].view(np.int16)).to(dev).view(tdt[dtype])
            w = torch.from_numpy(case["w"].view(np.int16)).to(dev).view(tdt[dtype])
        xs = [x0] + [x0.clone() for _ in range(sets - 1)]
        ys = [torch.empty_like(x0) for _ in range(sets)]
        fns = [binding.bind_rmsnorm_fwd(xs[i], w, ys[i], eps) for i in range(sets)]
        for i in range(10):
            fns[i % sets]()
        torch.cuda.synchronize()
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                 for _ in range(iters)]
        for i, (a, b) in enumerate(pairs):
            a.record()
            fns[i % sets]()
            b.record()
        torch.cuda.synchronize()
        us = trimmed_mean([a.elapsed_time(b) * 1e3 for a, b in pairs])
        sustained_us = timed_region(fns, iters) * 1e3
        t_all = min(_timed(lambda: oracle.rmsnorm_oracle(case["x"], case["w"], eps, dtype, cores))
                    for _ in range(3))
        rows1 = min(M, 512)
        t_one = min(_timed(lambda: oracle.rmsnorm_oracle(case["x"][:rows1], case["w"], eps, dtype, 1))
                    for _ in range(3)) * (M / rows1)
        entry = {
            "workload": case["name"], "bytes": nbytes, "buffer_sets": sets,
            "threads_per_row": binding.rmsnorm_auto_threads_per_row(N, dtype),
            "gpu_us": round(us, 2), "gpu_gbps": round(nbytes / us / 1e3, 1),
            "gpu_sustained_us": round(sustained_us, 2),
            "gpu_sustained_gbps": round(nbytes / sustained_us / 1e3, 1),
            "gpu_rows_per_s": round(M / us * 1e6, 1),
            "pct_of_peak": round(nbytes / us / 1e3 / PEAK_HBM_GBPS * 100, 2),
            "oracle_all_threads_s": round(t_all, 5), "oracle_threads": cores,
            "oracle_all_threads_gbps": round(nbytes / t_all / 1e9, 3),
            "oracle_one_thread_s_extrapolated": round(t_one, 4),
        }
        log(f"{entry}")
        out.append(entry)
        del xs, ys, fns
        torch.cuda.empty_cache()
    return out


def _timed(fn) -> float:
    t = time.perf_counter()
    fn()
    return time.perf_counter() - t


if __name__ == "__main__":
    sys.exit(main())
