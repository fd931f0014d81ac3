"""Sweep modes of bench.py: tables, not the one-line JSON contract.

  config2  block x R cells at n = 2^26 uniform [0,1) (Section 5.2's B x R
           experiment, on this GPU), both grid modes, + all-ones 2^24 exactness
  config5  n = 2^16 .. 2^30 and each 2^k + 7, MFMA kernel and shuffle kernel
  tune     geometry search at n = 2^28 (block, R, chains in flight, grid, load policy)
"""
from __future__ import annotations

import itertools
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
HBM_PEAK_GBPS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Timer:
    def __init__(self, torch, B):
        self.torch, self.B = torch, B
        self.stream = torch.cuda.current_stream().cuda_stream
        self.out = torch.zeros(8, dtype=torch.float32, device="cuda")

    def run(self, bufs, n, tuning, steps, warmup, offset_bytes=0):
        """Average seconds per call (HIP events around `steps` back-to-back calls)."""
        torch, B = self.torch, self.B
        k = len(bufs)
        ptrs = [b.data_ptr() + offset_bytes for b in bufs]
        for i in range(warmup):
            B.mfr_sum_f16_ex(ptrs[i % k], n, self.out.data_ptr(), tuning, self.stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            B.mfr_sum_f16_ex(ptrs[(warmup + i) % k], n, self.out.data_ptr(), tuning, self.stream)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / steps

    def result(self):
        self.torch.cuda.synchronize()
        return float(self.out[0].item())


def open_out(args, name):
    path = args.out or os.path.join(ROOT, "gpurun_out", name)
    os.makedirs(os.path.dirname(path), exist_ok=True)
    return open(path, "w")


def emit(f, line):
    print(line, flush=True)
    f.write(line + "\n")
    f.flush()


def device_buffers(torch, np, x, count):
    host = torch.from_numpy(x.view(np.int16))
    return [host.cuda() for _ in range(count)]


def heat(timer, bufs, n, seconds=1.0):
    """Keep the GPU busy so that clocks settle before anything is timed."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        timer.run(bufs, n, None, 50, 0)


def tune(args, torch, np, B, W):
    n = args.n
    x = W.generate("normal", n, W.config_seed(3))
    bufs = device_buffers(torch, np, x, args.buffers)
    timer = Timer(torch, B)
    heat(timer, bufs, n)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    rows = []
    with open_out(args, "tune.txt") as f:
        emit(f, "# n=%d buffers=%d CUs=%d ; columns: kernel block R U nt grid us GB/s pct" % (n, len(bufs), cus))
        combos = []
        for kernel in (0, 1):
            for block in (64, 128, 256, 512, 1024):
                for R, U in ((1, 1), (1, 2), (1, 4), (1, 8), (2, 1), (2, 2), (2, 4), (2, 8), (4, 1), (4, 2), (4, 4), (8, 1), (8, 2)):
                    waves = block // 64
                    if R * U * 1 < 2:
                        continue
                    for wpc in (1, 2, 4, 8, 16, 32):          # waves per CU
                        if wpc % waves:
                            continue
                        grid = cus * wpc // waves
                        for nt in (1, 2):
                            combos.append((kernel, block, R, U, nt, grid))
                    combos.append((kernel, block, R, U, 1, -1))
        if args.quick:
            combos = combos[::args.quick]
        for (kernel, block, R, U, nt, grid) in combos:
            t = B.make_tuning(block, R, grid, kernel, U, nt)
            dt = timer.run(bufs, n, t, args.steps, 5)
            gbps = 2 * n / dt / 1e9
            rows.append((gbps, kernel, block, R, U, nt, grid, dt))
            emit(f, "%d %4d %d %d %d %7d %8.2f %7.1f %5.1f" % (kernel, block, R, U, nt, grid, dt * 1e6, gbps, 100 * gbps / HBM_PEAK_GBPS))
        rows.sort(reverse=True)
        emit(f, "# best 25")
        for (gbps, kernel, block, R, U, nt, grid, dt) in rows[:25]:
            emit(f, "# %d %4d %d %d %d %7d %8.2f %7.1f %5.1f" % (kernel, block, R, U, nt, grid, dt * 1e6, gbps, 100 * gbps / HBM_PEAK_GBPS))


def run(args):
    import numpy as np
    import torch
    from paper_2001_05585_amd import binding as B
    from paper_2001_05585_amd import workloads as W
    if not torch.cuda.is_available():
        raise SystemExit("sweeps need a GPU")
    torch.cuda.set_device(0)
    B.lib()
    {"tune": tune}[args.sweep](args, torch, np, B, W)
