#!/usr/bin/env python3
"""Benchmark of libmfreduce on one MI355X.

Default run: the headline workload (config 3: n = 2^28 fp16 values, normal(0,1),
fp32 result), one "step" = one complete reduction (load, MFMA chains, block
combine, grid combine) of one resident 512 MiB buffer.  Several distinct
buffers are rotated so that the 256 MB last-level cache cannot serve the reads.
Prints ONE JSON line.

Other modes (they write tables to the results folder, not the JSON contract line):
  --sweep config2   block x R grid at n = 2^26 (+ all-ones 2^24 exactness)
  --sweep config5   n = 2^16 .. 2^30 (+7), MFMA kernel and shuffle kernel
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "Gelem/s and achieved HBM GB/s (% of peak) for fp16->fp32 sum, n=2^28, 1 GPU"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(n: int, grid: int) -> int:
    """2 bytes read per element, each block partial written and read once, the result written."""
    return 2 * n + (8 * grid if grid > 1 else 0) + 4


def make_buffers(torch, np, x, count):
    host = torch.from_numpy(x.view(np.int16))
    bufs = [host.cuda() for _ in range(count)]
    torch.cuda.synchronize()
    return bufs


PREHEAT_S = 0.25


def settle(torch, B, bufs, n, out, tuning, seconds):
    """Untimed calls on the rotating buffers for about `seconds`."""
    stream = torch.cuda.current_stream().cuda_stream
    k = len(bufs)
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(50):
            B.mfr_sum_f16_ex(bufs[i % k].data_ptr(), n, out.data_ptr(), tuning, stream)
            i += 1
        torch.cuda.synchronize()


def time_calls(torch, B, bufs, n, out, tuning, steps, warmup):
    """(wall seconds, event seconds) for `steps` back-to-back calls after `warmup` calls."""
    stream = torch.cuda.current_stream().cuda_stream
    k = len(bufs)
    for i in range(warmup):
        B.mfr_sum_f16_ex(bufs[i % k].data_ptr(), n, out.data_ptr(), tuning, stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        B.mfr_sum_f16_ex(bufs[(warmup + i) % k].data_ptr(), n, out.data_ptr(), tuning, stream)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return t1 - t0, e0.elapsed_time(e1) * 1e-3


def per_call_times(torch, B, bufs, n, out, tuning, steps):
    """Per-call durations (seconds) from one event pair per call."""
    stream = torch.cuda.current_stream().cuda_stream
    k = len(bufs)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(pairs):
        a.record()
        B.mfr_sum_f16_ex(bufs[i % k].data_ptr(), n, out.data_ptr(), tuning, stream)
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) * 1e-3 for a, b in pairs]


def cpu_baseline(x, n, gpu_value, budget_s=25.0):
    """The oracle as it stands, timed on the host cores (reported baseline, not a target)."""
    import oracle
    cores = min(os.cpu_count() or 1, 16)
    t0 = time.perf_counter()
    best_blocked, used, s, sa = None, cores, 0.0, 0.0
    for _ in range(3):
        a = time.perf_counter()
        s, sa, used = oracle.sum_f16_blocked(x, cores)
        dt = time.perf_counter() - a
        best_blocked = dt if best_blocked is None else min(best_blocked, dt)
    # definitional single-thread oracle on a bounded prefix (whole input if it fits the budget)
    m = n
    est = best_blocked * used
    if est > budget_s:
        m = max(1 << 20, int(n * budget_s / est))
    a = time.perf_counter()
    s1, sa1 = oracle.sum_f16(x[:m])
    single = time.perf_counter() - a
    res = {
        "value": round(n / best_blocked / 1e9, 4), "unit": "Gelem/s", "cores": int(used), "kind": "oracle",
        "sample": "whole workload (n=%d), fp64 Kahan oracle blocked over %d host threads, best of 3; "
                  "single-thread oracle on the first %d elements: %.4f Gelem/s" % (n, used, m, m / single / 1e9),
        "single_thread_gelems": round(m / single / 1e9, 4),
        "oracle_sum": s, "oracle_sum_abs": sa,
        "seconds_spent": round(time.perf_counter() - t0, 2),
    }
    if gpu_value is not None:
        ref = s1 if m == n else s
        err = abs(float(gpu_value) - ref)
        res["gpu_abs_err"] = err
        res["gpu_err_over_sum_abs"] = err / sa if sa else 0.0
        res["gpu_err_over_abs_sum"] = err / abs(ref) if ref else None
        res["within_1e-5_sum_abs"] = bool(err <= 1e-5 * sa)
    return res


TRAFFIC_RECORD = os.path.join("profiles", "hbm_traffic_sum_2p28.json")


def measured_traffic(n, tuning_is_default):
    """HBM bytes per launch from the recorded rocprofv3 --pmc runs (FETCH_SIZE / WRITE_SIZE) of this
    workload; None for any other size or geometry.  Counters cannot be read from inside this run."""
    if n != 1 << 28 or not tuning_is_default:
        return None
    try:
        with open(os.path.join(ROOT, TRAFFIC_RECORD)) as f:
            return json.load(f).get("bytes_per_launch")
    except (OSError, ValueError):
        return None


def headline(args):
    import numpy as np
    import torch
    from paper_2001_05585_amd import binding as B
    from paper_2001_05585_amd import workloads as W

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU: the HIP path has no fallback")
    torch.cuda.set_device(0)
    B.lib()
    n = args.n
    kind, cfg = ("normal", 3)
    log("generating %s n=%d ..." % (kind, n))
    x = W.generate(kind, n, W.config_seed(cfg))
    # enough distinct copies that the 256 MB last-level cache cannot serve the reads: 2 GiB in rotation
    copies = args.buffers if args.buffers > 0 else max(4, min(1024, (1 << 31) // max(2 * n, 1)))
    bufs = make_buffers(torch, np, x, copies)
    out = torch.zeros(4, dtype=torch.float32, device="cuda")
    tuning = B.make_tuning(args.block, args.R, args.grid, args.kernel, args.in_flight, args.nontemporal, args.combine)
    tuning_is_default = not any((args.block, args.R, args.grid, args.kernel, args.in_flight, args.nontemporal, args.combine))
    grid = B.mfr_grid_for(n, bufs[0].data_ptr(), None if tuning_is_default else tuning)
    if tuning_is_default:
        tuning = None              # the library's own choices, exactly as mfr_sum_f16 makes them
    log("timing: block=%d R=%d grid=%d kernel=%d, %d buffers ..." % (args.block, args.R, grid, args.kernel, copies))
    # Freshly allocated buffers run 3-10 % slow for their first few hundred calls: a quarter of a second
    # of untimed calls before the warm-up steps, so that short runs measure the sustained rate too.
    settle(torch, B, bufs, n, out, tuning, PREHEAT_S)
    wall, ev = time_calls(torch, B, bufs, n, out, tuning, args.steps, args.warmup)
    gpu_value = float(out[0].item())
    calls = per_call_times(torch, B, bufs, n, out, tuning, min(args.steps, 200))
    warm_wall, warm_ev = time_calls(torch, B, bufs[:1], n, out, tuning, args.steps, args.warmup)

    ms_per_step = wall / args.steps * 1e3
    value = n / (wall / args.steps) / 1e9
    launch_s = ev / args.steps
    nbytes = algorithmic_bytes(n, grid)
    achieved = nbytes / launch_s / 1e9
    b, r, g = B.mfr_get_default_tuning()
    result = {
        "metric": METRIC, "value": round(value, 3), "unit": "Gelem/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: sum of n=%d fp16 values i.i.d. normal(0,1), fp32 result; "
                               "%d distinct %.4g MiB buffers rotated" % ("config 3" if n == 1 << 28 else "config 3's distribution at another size",
                                                                        n, len(bufs), 2 * n / 2 ** 20),
                   "n": n, "input_dtype": "f16", "kernel": ("mfma_chain", "shfl_tree", "split")[args.kernel],
                   "block_threads": args.block or b, "chain_R": args.R or r,
                   "grid_blocks": grid, "buffers": len(bufs), "untimed_preheat_s": PREHEAT_S},
        "hbm_gbps": round(achieved, 1), "pct_hbm_peak": round(100 * achieved / HBM_PEAK_GBPS, 2),
        "per_call_us": {"median": round(statistics.median(calls) * 1e6, 2), "min": round(min(calls) * 1e6, 2)},
        "single_buffer": {"gelems": round(n / (warm_wall / args.steps) / 1e9, 3),
                          "hbm_gbps": round(nbytes / (warm_ev / args.steps) / 1e9, 1),
                          "note": "one buffer re-read; part of it is served by the last-level cache"},
        "paper_context": "paper reports ~3.2x over a conventional GPU reduction on Nvidia tensor-core hardware",
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(n, tuning_is_default),
                     "traffic_source": ("recorded rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE runs of this workload (%s), "
                                        "not measured in this run" % TRAFFIC_RECORD) if measured_traffic(n, tuning_is_default) is not None else None,
                     "kernel": "sum_kernel", "bytes_per_launch": nbytes,
                     "launch_us": round(launch_s * 1e6, 3)},
    }
    if not args.no_cpu_baseline:
        log("cpu baseline (oracle) ...")
        result["cpu_baseline"] = cpu_baseline(x, n, gpu_value)
    print(json.dumps(result), flush=True)


def traffic(args):
    """A short run for `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`: a few launches of the
    sum kernel on rotating buffers, and a plain elementwise copy of the same 512 MiB (reads n*2
    bytes, writes n*2 bytes) whose counter reading calibrates the unit of the counters."""
    import numpy as np
    import torch
    from paper_2001_05585_amd import binding as B
    from paper_2001_05585_amd import workloads as W
    torch.cuda.set_device(0)
    n = args.n
    x = W.generate("normal", n, W.config_seed(3))
    bufs = make_buffers(torch, np, x, args.buffers if args.buffers > 0 else 4)
    dst = torch.empty_like(bufs[0])
    out = torch.zeros(4, dtype=torch.float32, device="cuda")
    tuning = B.make_tuning(args.block, args.R, args.grid, args.kernel, args.in_flight, args.nontemporal, args.combine)
    stream = torch.cuda.current_stream().cuda_stream
    for i in range(args.steps):
        B.mfr_sum_f16_ex(bufs[i % len(bufs)].data_ptr(), n, out.data_ptr(), tuning, stream)
    torch.cuda.synchronize()
    for i in range(4):
        torch.mul(bufs[i % len(bufs)], 1, out=dst)       # elementwise copy kernel of known size
    torch.cuda.synchronize()
    print(json.dumps({"mode": "traffic", "n": n, "sum_launches": args.steps, "copy_launches": 4,
                      "copy_bytes_read": 2 * n, "copy_bytes_written": 2 * n, "result": float(out[0].item())}))


ROWS_TRAFFIC_SHAPES = (
    # (dtype name, cols, stride, shift in elements); rows fill 512 MiB
    ("f16", 32, 32, 0), ("f16", 64, 64, 0), ("f16", 100, 100, 0), ("f16", 256, 256, 0), ("f16", 1001, 1001, 0),
    ("f16", 1024, 1024, 0), ("f16", 4096, 4096, 0), ("f16", 256, 256, 1), ("f32", 256, 256, 0),
    # rows a few bytes longer than a whole number of steps, and 32-byte rows
    ("f16", 257, 257, 0), ("f16", 514, 514, 0), ("f16", 1030, 1030, 0), ("f16", 16, 16, 0),
    # a single masked step that is little more than half full; rows 2 bytes off a 4-byte boundary
    ("f16", 300, 300, 0), ("f16", 500, 500, 1),
)


def traffic_rows(args):
    """The same kind of run for the many-rows kernel: each shape four times on rotating buffers, in
    the order of ROWS_TRAFFIC_SHAPES, then the calibration copy."""
    import numpy as np
    import torch
    from paper_2001_05585_amd import binding as B
    from paper_2001_05585_amd import workloads as W
    torch.cuda.set_device(0)
    n = 1 << 28
    x = W.generate("normal", n, W.config_seed(3))
    bufs = make_buffers(torch, np, x, 4)
    dst = torch.empty_like(bufs[0])
    out = torch.zeros((1 << 24) + 8, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    shapes = []
    for name, cols, stride, shift in ROWS_TRAFFIC_SHAPES:
        dtype, esize = (B.MFR_DTYPE_F32, 4) if name == "f32" else (B.MFR_DTYPE_F16, 2)
        rows = (2 * n // esize) // stride - (1 if shift else 0)
        for i in range(4):
            B.mfr_sum_rows_ex(bufs[i].data_ptr() + shift * esize, dtype, rows, cols, stride, out.data_ptr(), None, stream)
        torch.cuda.synchronize()
        shapes.append({"type": name, "rows": rows, "cols": cols, "stride": stride, "shift": shift, "launches": 4,
                       "bytes_read": rows * cols * esize, "bytes_written": rows * 4})
    for i in range(4):
        torch.mul(bufs[i % len(bufs)], 1, out=dst)       # elementwise copy kernel of known size
    torch.cuda.synchronize()
    print(json.dumps({"mode": "traffic-rows", "shapes": shapes, "copy_launches": 4, "copy_bytes_read": 2 * n,
                      "copy_bytes_written": 2 * n}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--n", type=int, default=1 << 28)
    ap.add_argument("--buffers", type=int, default=0, help="distinct input copies in rotation (0: 2 GiB worth, at least 4)")
    ap.add_argument("--block", type=int, default=0)
    ap.add_argument("--R", type=int, default=0)
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0)
    ap.add_argument("--in-flight", type=int, default=0)
    ap.add_argument("--nontemporal", type=int, default=0)
    ap.add_argument("--combine", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic", action="store_true", help="short run for rocprofv3 --pmc counters")
    ap.add_argument("--traffic-rows", action="store_true", help="the same for the many-rows kernel")
    ap.add_argument("--sweep", choices=["config2", "config5", "types", "rows", "row_lengths", "split", "variants", "wide", "timeline"], default=None)
    ap.add_argument("--quick", type=int, default=0, help="sweeps: keep every k-th combination")
    ap.add_argument("--out", default=None, help="file for sweep tables (default: <results folder>/<sweep>.txt)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (--gpus 1); the reduction shards trivially "
                         "but no multi-GPU path is part of it")
    from paper_2001_05585_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):     # load what is built; build only if nothing is
        build.build()
    if args.traffic:
        traffic(args)
    elif args.traffic_rows:
        traffic_rows(args)
    elif args.sweep:
        import bench_sweeps
        bench_sweeps.run(args)
    else:
        headline(args)


if __name__ == "__main__":
    main()
