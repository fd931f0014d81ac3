"""Sweep modes of bench.py: tables, not the one-line JSON contract.

  config2  block x R cells at n = 2^26 uniform [0,1) (Section 5.2's B x R
           experiment, on this GPU), both grid modes, + all-ones 2^24 exactness
  config5  n = 2^16 .. 2^30 and each 2^k + 7, MFMA kernel and shuffle kernel
  types    512 MiB of binary16 / bfloat16 / binary32 through both kernels
  rows     batched form: rows x cols filling 512 MiB, and a walk over row lengths
  split    Section 5.3's fraction experiment
  variants Section 5.4's run time and error of the variants over n
  wide     the binary64-accumulation mode beside the fp32 mode
  timeline where the time of a call goes, from the kernel's own clock readings
"""
from __future__ import annotations

import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
RESULTS_DIR = os.environ.get("MFR_RESULTS_DIR", os.path.join(ROOT, "gpurun_out"))
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


def rows_shape_label(plan):
    """Name of a many-rows kernel shape as mfr_rows_plan reports it."""
    label = "P%d_D%d_GF%d" % (plan[0], plan[1], plan[2])
    label += "_tail%d" % (1 << (plan[11] >> 2)) if plan[11] & 1 else ("" if plan[9] else "_masked")
    return label + ("_shifted" if plan[11] & 2 else "")


def oracle_reference(x):
    """(sum, sum of |x|) of the fp16 array x from the CPU oracle, blocked over the host cores: the
    checking leg of the sweeps (every timed cell is also compared with it); nothing else here uses
    the oracle."""
    import oracle
    s, sa, _ = oracle.sum_f16_blocked(x, min(os.cpu_count() or 1, 16))
    return s, sa


def rel_err(value, ref):
    s, sa = ref
    return abs(float(value) - s) / sa if sa else 0.0


def load_context():
    """ctypes handle of the hipCUB comparison library, or None if it has not been built."""
    import ctypes
    path = os.path.join(ROOT, "paper_2001_05585_amd", "libmfrcontext.so")
    if not os.path.exists(path):
        return None
    lib = ctypes.CDLL(path)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    for name in ("ctx_hipcub_sum_f16_f32acc", "ctx_hipcub_sum_f16"):
        fn = getattr(lib, name)
        fn.argtypes = [vp, sz, vp, vp, ctypes.POINTER(sz), vp]
        fn.restype = ctypes.c_int
    return lib


def open_out(args, name):
    path = args.out or os.path.join(RESULTS_DIR, name)
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


def arena_pointers(base_ptr, arena_bytes, n, max_count=4096):
    """Distinct, 256-byte aligned starting addresses for n-element inputs inside one arena."""
    stride = (2 * n + 255) // 256 * 256
    count = max(1, min(max_count, arena_bytes // stride))
    return [base_ptr + i * stride for i in range(count)]


def time_rotating(timer, ptrs, n, tuning, steps, warmup):
    torch, B = timer.torch, timer.B
    k = len(ptrs)
    for i in range(warmup):
        B.mfr_sum_f16_ex(ptrs[i % k], n, timer.out.data_ptr(), tuning, timer.stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        B.mfr_sum_f16_ex(ptrs[(warmup + i) % k], n, timer.out.data_ptr(), tuning, timer.stream)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / steps


def config2(args, torch, np, B, W):
    """Block x R cells (Section 5.2's configuration experiment) at n = 2^26, uniform [0,1)."""
    n = args.n if args.n != 1 << 28 else 1 << 26     # --n overrides (e.g. 2^20, the size of the paper's experiment)
    x = W.generate("uniform01", n, W.config_seed(2))
    copies = max(16, min(512, (1 << 31) // (2 * n)))  # 2 GiB in rotation: the last-level cache cannot hold it
    bufs = device_buffers(torch, np, x, copies)
    ptrs = [b.data_ptr() for b in bufs]
    ones = torch.ones(1 << 24, dtype=torch.float16, device="cuda")
    timer = Timer(torch, B)
    ref = oracle_reference(x)
    heat(timer, bufs, n)
    with open_out(args, "config2.txt") as f:
        emit(f, "# config 2: n=%d uniform[0,1), MFMA-chain kernel; rotating %d x %.3f MiB buffers (cold) and one buffer (warm, cache-resident)" % (n, copies, 2 * n / 2 ** 20))
        emit(f, "# grid: persistent = MFR_GRID_AUTO, one-chain = one chain of R MFMAs per wave (the paper's geometry)")
        emit(f, "# err/sum|x| = |gpu - oracle| / sum|x_i| of the timed cell's result against the fp64 Kahan oracle (gate: 1e-5)")
        emit(f, "# block R grid_mode blocks cold_us cold_Gelem/s cold_GB/s cold_pct warm_us warm_GB/s err/sum|x| ones_2p24")
        for grid_mode, gname in ((B.MFR_GRID_AUTO, "persistent"), (B.MFR_GRID_ONE_CHAIN, "one-chain")):
            for block in (32, 64, 128, 256, 512, 1024):
                for R in range(1, 9):
                    t = B.make_tuning(block, R, grid_mode)
                    steps = args.steps if grid_mode == B.MFR_GRID_AUTO else max(5, args.steps // 4)
                    cold = time_rotating(timer, ptrs, n, t, steps, 3)
                    warm = time_rotating(timer, ptrs[:1], n, t, steps, 3)
                    err = rel_err(timer.result(), ref)
                    if not err <= 1e-5:
                        raise SystemExit("config2: block %d R %d %s: |err|/sum|x| = %g" % (block, R, gname, err))
                    B.mfr_sum_f16_ex(ones.data_ptr(), 1 << 24, timer.out.data_ptr(), t, timer.stream)
                    exact = "exact" if timer.result() == 16777216.0 else "WRONG(%r)" % timer.result()
                    label = "32(wave64,half-filled)" if block == 32 else str(block)
                    emit(f, "%s %d %s %d %.2f %.1f %.1f %.1f %.2f %.1f %.2e %s" % (
                        label, R, gname, B.mfr_grid_for(n, ptrs[0], t), cold * 1e6, n / cold / 1e9,
                        2 * n / cold / 1e9, 100 * 2 * n / cold / 1e9 / HBM_PEAK_GBPS, warm * 1e6, 2 * n / warm / 1e9, err, exact))


def config5(args, torch, np, B, W):
    """n = 2^16 .. 2^30 and each 2^k + 7; MFMA-chain kernel and shuffle-tree kernel, default tuning."""
    nmax = (1 << 30) + 7
    x = W.generate("uniform01", nmax, W.config_seed(5))
    arena = torch.from_numpy(x.view(np.int16)).cuda()
    arena_bytes = 2 * nmax
    timer = Timer(torch, B)
    ctx = load_context()
    heat(timer, [arena], 1 << 28)
    with open_out(args, "config5.txt") as f:
        emit(f, "# config 5: uniform[0,1); inputs rotate through a 2 GiB arena (distinct addresses per call) so that")
        emit(f, "# sizes below the last-level cache capacity are not served from cache; default tuning per kernel")
        emit(f, "# err/sum|x| = |gpu - oracle| / sum|x_i| against the fp64 Kahan oracle on the first of the rotating slices (gate: 1e-5);")
        emit(f, "# mfma_chain = the library's default entry (t == NULL), shfl_tree = the conventional kernel with default tuning")
        emit(f, "# n kernel blocks us Gelem/s GB/s pct_of_8TB/s err/sum|x|")
        for k in range(16, 31):
            for n in (1 << k, (1 << k) + 7):
                ptrs = arena_pointers(arena.data_ptr(), arena_bytes, n)
                ref = oracle_reference(x[:n])
                for kernel, kname in ((B.MFR_KERNEL_MFMA, "mfma_chain"), (B.MFR_KERNEL_SHFL, "shfl_tree")):
                    t = None if kernel == B.MFR_KERNEL_MFMA else B.make_tuning(kernel=kernel)
                    steps = max(10, min(args.steps * 4, int(2e-2 / max(2 * n / 6e12, 4e-6))))
                    dt = time_rotating(timer, ptrs, n, t, steps, 5)
                    B.mfr_sum_f16_ex(ptrs[0], n, timer.out.data_ptr(), t, timer.stream)
                    err = rel_err(timer.result(), ref)
                    if not err <= 1e-5:
                        raise SystemExit("config5: n %d %s: |err|/sum|x| = %g" % (n, kname, err))
                    emit(f, "%d %s %d %.2f %.2f %.1f %.2f %.2e" % (n, kname, B.mfr_grid_for(n, ptrs[0], t), dt * 1e6,
                                                                 n / dt / 1e9, 2 * n / dt / 1e9, 100 * 2 * n / dt / 1e9 / HBM_PEAK_GBPS, err))
                # context only: PyTorch's own reduction (fp32 accumulation) on the same rotating slices
                halves = arena.view(torch.float16)
                stride_e = (ptrs[1] - ptrs[0]) // 2 if len(ptrs) > 1 else 0
                views = [halves[i * stride_e:i * stride_e + n] for i in range(len(ptrs))]
                steps = max(10, min(args.steps * 4, int(2e-2 / max(2 * n / 6e12, 4e-6))))
                for i in range(5):
                    torch.sum(views[i % len(views)], dtype=torch.float32)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(steps):
                    torch.sum(views[(i + 5) % len(views)], dtype=torch.float32)
                e1.record()
                torch.cuda.synchronize()
                dt = e0.elapsed_time(e1) * 1e-3 / steps
                emit(f, "%d %s %d %.2f %.2f %.1f %.2f" % (n, "torch.sum(context)", 0, dt * 1e6, n / dt / 1e9, 2 * n / dt / 1e9,
                                                        100 * 2 * n / dt / 1e9 / HBM_PEAK_GBPS))
                # context only: the vendor's device-wide reduction (hipCUB), float and half accumulation
                if ctx is not None:
                    import ctypes
                    for fname, label in (("ctx_hipcub_sum_f16_f32acc", "hipcub_float_acc(context)"), ("ctx_hipcub_sum_f16", "hipcub_half_acc(context)")):
                        fn = getattr(ctx, fname)
                        need = ctypes.c_size_t(0)
                        fn(ptrs[0], n, timer.out.data_ptr(), None, ctypes.byref(need), timer.stream)
                        temp = torch.empty(max(int(need.value), 256), dtype=torch.uint8, device="cuda")
                        for i in range(5):
                            fn(ptrs[i % len(ptrs)], n, timer.out.data_ptr(), temp.data_ptr(), ctypes.byref(need), timer.stream)
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        for i in range(steps):
                            fn(ptrs[(i + 5) % len(ptrs)], n, timer.out.data_ptr(), temp.data_ptr(), ctypes.byref(need), timer.stream)
                        e1.record()
                        torch.cuda.synchronize()
                        dt = e0.elapsed_time(e1) * 1e-3 / steps
                        emit(f, "%d %s %d %.2f %.2f %.1f %.2f" % (n, label, 0, dt * 1e6, n / dt / 1e9, 2 * n / dt / 1e9,
                                                                100 * 2 * n / dt / 1e9 / HBM_PEAK_GBPS))


def types(args, torch, np, B, W):
    """512 MiB of each element type through both kernels (default tuning), rotating 4 buffers."""
    timer = Timer(torch, B)
    with open_out(args, "types.txt") as f:
        emit(f, "# 512 MiB per call, normal(0,1), 4 rotating buffers, default tuning, 0.5 s of calls before the timed ones; GB/s = bytes / time")
        emit(f, "# dtype n kernel us Gelem/s GB/s pct_of_8TB/s")
        for dtype, name, esize in ((B.MFR_DTYPE_F16, "f16", 2), (B.MFR_DTYPE_BF16, "bf16", 2), (B.MFR_DTYPE_F32, "f32", 4)):
            n = (1 << 29) // esize
            if dtype == B.MFR_DTYPE_F16:
                host = torch.from_numpy(W.generate("normal", n, 3).view(np.int16))
            elif dtype == B.MFR_DTYPE_BF16:
                host = torch.from_numpy(W.generate_bf16("normal", n, 3).view(np.int16))
            else:
                host = torch.from_numpy(W.generate_f32("normal", n, 3))
            bufs = [host.cuda() for _ in range(4)]
            # binary32: three of four additions are vector-ALU adds in the lane, one MFMA per tile adds the lanes
            for kernel, kname in ((B.MFR_KERNEL_MFMA, "valu+mfma_chain" if dtype == B.MFR_DTYPE_F32 else "mfma_chain"),
                                  (B.MFR_KERNEL_SHFL, "shfl_tree")):
                t = B.make_tuning(kernel=kernel)

                def call(i):
                    B.mfr_sum_ex(bufs[i % 4].data_ptr(), dtype, n, timer.out.data_ptr(), t, timer.stream)
                # freshly allocated buffers run slow at first: half a second of calls before the timed ones
                t0 = time.perf_counter()
                while time.perf_counter() - t0 < 0.5:
                    for i in range(50):
                        call(i)
                    torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(args.steps):
                    call(i)
                e1.record()
                torch.cuda.synchronize()
                dt = e0.elapsed_time(e1) * 1e-3 / args.steps
                gb = n * esize / dt / 1e9
                emit(f, "%s %d %s %.2f %.1f %.1f %.1f" % (name, n, kname, dt * 1e6, n / dt / 1e9, gb, 100 * gb / HBM_PEAK_GBPS))
            del bufs


def split(args, torch, np, B, W):
    """Section 5.3's experiment: fraction of the domain through the MFMA path vs the conventional path."""
    timer = Timer(torch, B)
    with open_out(args, "split.txt") as f:
        emit(f, "# split variant: permille of the domain (and of the waves) on the MFMA path; fp16 normal(0,1)")
        emit(f, "# n residency block R U grid permille_mfma us Gelem/s GB/s")
        for n, copies, label in ((1 << 28, 4, "HBM(4x512MiB rotating)"), (1 << 24, 1, "cache-resident(32MiB)")):
            x = W.generate("normal", n, W.config_seed(3))
            bufs = device_buffers(torch, np, x, copies)
            heat(timer, bufs, n, 0.3)
            for block, R, U, grid in ((256, 4, 2, 0), (256, 1, 8, 0), (1024, 1, 2, 2048), (256, 1, 2, 2048)):
                for pm in (0, 100, 250, 400, 500, 600, 750, 900, 1000):
                    t = B.make_tuning(block, R, grid, B.MFR_KERNEL_SPLIT, U, 0, 0, pm)
                    dt = timer.run(bufs, n, t, args.steps, 5)
                    emit(f, "%d %s %d %d %d %d %d %.2f %.1f %.1f" % (n, label, block, R, U, B.mfr_grid_for(n, bufs[0].data_ptr(), t),
                                                                  pm, dt * 1e6, n / dt / 1e9, 2 * n / dt / 1e9))
            del bufs


def variants(args, torch, np, B, W):
    """Section 5.4's comparison on this GPU: run time of the single-pass, recurrence and shuffle
    kernels and the result each returns, over n, for normal(0,1) and uniform[0,1) inputs.
    The error columns are Section 5.4's "% error against a CPU reduction in double precision",
    100 |gpu - oracle| / |oracle|, and |gpu - oracle| / sum|x_i| (the figure the tolerance is stated in)."""
    timer = Timer(torch, B)
    out = torch.zeros(4, dtype=torch.float32, device="cuda")
    with open_out(args, "variants.txt") as f:
        emit(f, "# one buffer per n (sizes up to 2^26 are cache-resident); inf = the variant's binary16 partials overflowed")
        emit(f, "# kind n variant us Gelem/s result err_pct_of_|sum| err/sum|x|")
        for kind, cfg in (("normal", 3), ("uniform01", 2)):
            x = W.generate(kind, 1 << 28, W.config_seed(cfg))
            dev = torch.from_numpy(x.view(np.int16)).cuda()
            for k in range(10, 29, 2):
                n = 1 << k
                ref = oracle_reference(x[:n])
                calls = (("single_pass", lambda: B.mfr_sum_f16(dev.data_ptr(), n, out.data_ptr(), timer.stream)),
                         ("recurrence_R4", lambda: B.mfr_sum_f16_recurrence(dev.data_ptr(), n, out.data_ptr(), 4, timer.stream)),
                         ("recurrence_R5", lambda: B.mfr_sum_f16_recurrence(dev.data_ptr(), n, out.data_ptr(), 5, timer.stream)),
                         ("shuffle_tree", lambda: B.mfr_sum_f16_tuned(dev.data_ptr(), n, out.data_ptr(), 256, 4, 0, 1, timer.stream)))
                for name, call in calls:
                    for _ in range(5):
                        call()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(args.steps):
                        call()
                    e1.record()
                    torch.cuda.synchronize()
                    dt = e0.elapsed_time(e1) * 1e-3 / args.steps
                    got = float(out[0].item())
                    pct = 100.0 * abs(got - ref[0]) / abs(ref[0]) if ref[0] else float("nan")
                    emit(f, "%s %d %s %.2f %.2f %r %.3g %.3g" % (kind, n, name, dt * 1e6, n / dt / 1e9, got, pct, rel_err(got, ref)))


def wide(args, torch, np, B, W):
    """Run time of the binary64-accumulation mode beside the standard fp32 mode at n = 2^28."""
    n = 1 << 28
    x = W.generate("uniform01", n, W.config_seed(2))
    bufs = device_buffers(torch, np, x, 4)
    timer = Timer(torch, B)
    out64 = torch.zeros(2, dtype=torch.float64, device="cuda")
    heat(timer, bufs, n, 0.5)
    with open_out(args, "wide.txt") as f:
        emit(f, "# n=2^28 uniform[0,1), 4 rotating buffers; mode R U us Gelem/s GB/s pct_of_8TB/s result")
        dt = timer.run(bufs, n, None, args.steps, 10)
        emit(f, "fp32_partials 3 2 %.2f %.1f %.1f %.1f %r" % (dt * 1e6, n / dt / 1e9, 2 * n / dt / 1e9, 100 * 2 * n / dt / 1e9 / HBM_PEAK_GBPS, timer.result()))
        for R, U in ((1, 6), (1, 8), (2, 3), (2, 4), (3, 2), (4, 2), (6, 1), (8, 1)):
            t = B.make_tuning(256, R, 0, 0, U)

            def call(i):
                B.mfr_sum_f16_f64_ex(bufs[i % 4].data_ptr(), n, out64.data_ptr(), t, timer.stream)
            for i in range(10):
                call(i)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(args.steps):
                call(i)
            e1.record()
            torch.cuda.synchronize()
            dt = e0.elapsed_time(e1) * 1e-3 / args.steps
            emit(f, "binary64_after_chain %d %d %.2f %.1f %.1f %.1f %r" % (R, U, dt * 1e6, n / dt / 1e9, 2 * n / dt / 1e9,
                                                                      100 * 2 * n / dt / 1e9 / HBM_PEAK_GBPS, float(out64[0].item())))


def rows(args, torch, np, B, W):
    """Batched form: rows x cols elements filling 512 MiB per call, 4 rotating buffers."""
    total_bytes = 1 << 29
    host = torch.from_numpy(W.generate("normal", total_bytes // 2, 3).view(np.int16))
    bufs = [host.cuda() for _ in range(4)]
    timer = Timer(torch, B)
    out = torch.zeros(1 << 23, dtype=torch.float32, device="cuda")
    explicit = B.make_tuning()           # all defaults, but explicit: the per-row kernels
    names = {B.MFR_DTYPE_F16: "f16", B.MFR_DTYPE_BF16: "bf16", B.MFR_DTYPE_F32: "f32"}

    def measure(f, dtype, r, c, stride, shift_elems, t, label):
        esize = 4 if dtype == B.MFR_DTYPE_F32 else 2
        off = shift_elems * esize

        def call(i):
            B.mfr_sum_rows_ex(bufs[i % 4].data_ptr() + off, dtype, r, c, stride, out.data_ptr(), t, timer.stream)
        for i in range(5):
            call(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.steps):
            call(i)
        e1.record()
        torch.cuda.synchronize()
        dt = e0.elapsed_time(e1) * 1e-3 / args.steps
        gb = (esize * r * c + 4 * r) / dt / 1e9
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        plan = B.mfr_rows_plan(bufs[0].data_ptr() + off, dtype, r, c, stride, cus)
        if t is not None or plan is None:
            g = B.mfr_rows_geometry(bufs[0].data_ptr() + off, dtype, r, c, stride, t, cus)
            shape = "per-row_%dx%d_R%dU%d%s%s" % (g[0], g[1], g[2], g[3], "_staggered" if g[5] else "", "_limited" if g[6] else "")
        else:
            shape = rows_shape_label(plan)
        emit(f, "%s %d %d %d %d %s %s %.2f %.1f %.1f %.1f" % (names[dtype], r, c, stride, shift_elems, label, shape, dt * 1e6,
                                                       r * c / dt / 1e9, gb, 100 * gb / HBM_PEAK_GBPS))

    heat(timer, bufs, total_bytes // 2, 0.5)         # fresh buffers start slow
    with open_out(args, "rows.txt") as f:
        emit(f, "# rows x cols filling 512 MiB per call, 4 rotating buffers; 'default' = library choice (t == NULL), 'explicit' = the")
        emit(f, "# same call with an explicit all-default tuning, which selects the per-row kernels; shift = elements between a")
        emit(f, "# 16-byte boundary and x; GB/s counts the input and the 4-byte results")
        emit(f, "# kernel_shape of the per-row kernels: threads per block x blocks per row, chain_R, chains in flight, whether the rows")
        emit(f, "# start staggered and whether unused LDS limits the blocks resident per compute unit")
        emit(f, "# type rows cols stride shift tuning kernel_shape us Gelem/s GB/s pct_of_8TB/s")
        f16 = B.MFR_DTYPE_F16
        total = total_bytes // 2
        for lr in (0, 1, 2, 3, 4, 5, 6, 8, 9, 10, 11, 12, 14, 16, 17, 18, 19, 20, 21, 22, 23):
            r, c = 1 << lr, total >> lr
            measure(f, f16, r, c, c, 0, None, "default")
            if lr >= 4 and args.quick != 2:
                measure(f, f16, r, c, c, 0, explicit, "explicit")
            if lr >= 5:
                measure(f, f16, r - 1, c, c, 1, None, "default")
        for c, stride in ((100, 100), (100, 104), (300, 300), (384, 384), (600, 600), (768, 768), (1000, 1000), (1001, 1001), (2049, 2049), (2304, 2304), (3000, 3000), (4104, 4104),
                          (5000, 5000), (5001, 5001), (7000, 7000), (8192, 8192), (50000, 50001),
                          (50002, 50002), (268425, 268425), (268426, 268426), (16777209, 16777209), (16777210, 16777210)):
            r = total // stride
            measure(f, f16, r, c, stride, 0, None, "default")
        # row counts that are no power of two: a few hundred rows leave SIMDs without a wave
        for r in (100, 300, 400, 450, 520, 600, 700, 800, 900, 1030, 1100, 1400, 1500, 1800, 3000):
            c = total // r // 8 * 8
            measure(f, f16, r, c, c, 0, None, "default")
        for r in (300, 520, 600, 700, 1100, 1400):
            c = total // 2 // r // 8 * 8
            measure(f, B.MFR_DTYPE_F32, r, c, c, 0, None, "default")
        # row pitches that put unstaggered rows onto the same memory channels, and 1500 rows of 80 KB
        for r, c in ((145, 1851272), (143, 1877168), (339, 791840), (1024, 260144), (1500, 40000)):
            measure(f, f16, r, c, c, 0, None, "default")
        for r, c in ((113, 1187764), (1024, 130072)):
            measure(f, B.MFR_DTYPE_F32, r, c, c, 0, None, "default")
        for dtype in (B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32):
            esize = 4 if dtype == B.MFR_DTYPE_F32 else 2
            n = total_bytes // esize
            for c in (32, 64, 256, 1024, 4096, 1001):
                measure(f, dtype, n // c, c, c, 0, None, "default")
            measure(f, dtype, n // 256 - 1, 256, 256, 1, None, "default")


def row_lengths(args, torch, np, B, W):
    """Batched form over a fine grid of row lengths (contiguous rows filling 512 MiB, library defaults):
    shows which kernel shape each length gets and what it reaches."""
    total_bytes = 1 << 29
    host = torch.from_numpy(W.generate("normal", total_bytes // 2, 3).view(np.int16))
    bufs = [host.cuda() for _ in range(4)]
    timer = Timer(torch, B)
    out = torch.zeros((1 << 24) + 8, dtype=torch.float32, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    byte_lengths = [32, 48, 64, 96, 128, 160, 192, 200, 256, 320, 384, 400, 512, 514, 520, 576, 580, 600, 700, 768, 800, 900, 1000, 1022,
                    1024, 1028, 1040, 1088, 1200, 1280, 1400, 1434, 1536, 1540, 1600, 1800, 2000, 2048, 2060, 2112, 2200, 2560, 2800, 3000,
                    3072, 3500, 4000, 4096, 4104, 4608, 5000, 6000, 6144, 7000, 8192, 8208, 10000, 12288, 14000, 16384, 20000, 32768]
    heat(timer, bufs, total_bytes // 2, 0.5)         # fresh buffers start slow
    with open_out(args, "row_lengths.txt") as f:
        emit(f, "# contiguous rows filling 512 MiB per call, 4 rotating buffers, library defaults; GB/s counts the input and the 4-byte results")
        emit(f, "# f16+2: the same binary16 rows with the array starting 2 bytes off a 16-byte boundary (rows of an even number of")
        emit(f, "# elements then all start 2 bytes off a 4-byte boundary)")
        emit(f, "# type row_bytes cols rows kernel_shape steps_per_row us GB/s pct_of_8TB/s")
        off2_lengths = [32, 64, 128, 200, 256, 300, 400, 512, 600, 700, 768, 1000, 1024, 1032, 1500, 2048, 2100, 3000, 4000, 4096, 6000, 8192]
        for name, dtype, esize, first_byte in (("f16", B.MFR_DTYPE_F16, 2, 0), ("f32", B.MFR_DTYPE_F32, 4, 0), ("f16+2", B.MFR_DTYPE_F16, 2, 2)):
            for nbytes in (off2_lengths if first_byte else byte_lengths):
                if nbytes % esize:
                    continue
                c = nbytes // esize
                r = (total_bytes - first_byte) // nbytes
                if r + 8 > out.numel():
                    continue

                def call(i):
                    B.mfr_sum_rows_ex(bufs[i % 4].data_ptr() + first_byte, dtype, r, c, c, out.data_ptr(), None, timer.stream)
                for i in range(20):
                    call(i)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(args.steps):
                    call(i)
                e1.record()
                torch.cuda.synchronize()
                dt = e0.elapsed_time(e1) * 1e-3 / args.steps
                gb = (esize * r * c + 4 * r) / dt / 1e9
                plan = B.mfr_rows_plan(bufs[0].data_ptr() + first_byte, dtype, r, c, c, cus)
                if plan is None:
                    g = B.mfr_rows_geometry(bufs[0].data_ptr() + first_byte, dtype, r, c, c, None, cus)
                    shape = "per-row_%dx%d_R%dU%d%s" % (g[0], g[1], g[2], g[3], "_limited" if g[6] else "")
                else:
                    shape = rows_shape_label(plan)
                emit(f, "%s %d %d %d %s %s %.2f %.1f %.1f" % (name, nbytes, c, r, shape, "-" if plan is None else plan[4], dt * 1e6, gb,
                                                         100 * gb / HBM_PEAK_GBPS))


def timeline(args, torch, np, B, W):
    """Where the time of a call goes, from the kernel's own clock readings (mfr_sum_f16_stamped): for each
    size the call period without stamps (HIP events over back-to-back calls on rotating inputs), and, from
    20 stamped calls, the spread of the block starts, when the first and the last block had consumed its
    last chain, when the last partial was handed over and when the result was stored, all counted from the
    first block's start."""
    nmax = 1 << 30
    x = W.generate("uniform01", nmax, W.config_seed(5))
    arena = torch.from_numpy(x.view(np.int16)).cuda()
    timer = Timer(torch, B)
    heat(timer, [arena], 1 << 28)
    tick_us = 1e3 / B.mfr_wall_clock_khz()
    with open_out(args, "timeline.txt") as f:
        emit(f, "# uniform[0,1), library defaults (t == NULL), inputs rotating through a 2 GiB arena; times in us")
        emit(f, "# period = HIP events over back-to-back unstamped calls; the other columns are means over 20 stamped calls,")
        emit(f, "# counted from the start of the first block: spread of the block starts, first / last block done with its chains,")
        emit(f, "# last partial handed over, result stored; ideal = 2 n bytes at 8 TB/s")
        emit(f, "# n blocks period start_spread first_streamed last_streamed last_handed_over stored ideal_8TB/s")
        notes = []
        for k in (16, 18, 20, 22, 23, 24, 25, 26, 27, 28, 29, 30):
            n = 1 << k
            ptrs = arena_pointers(arena.data_ptr(), 2 * nmax, n)
            grid = B.mfr_grid_for(n, ptrs[0], None)
            steps = max(20, min(400, int(2e-2 / max(2 * n / 6e12, 4e-6))))
            period = time_rotating(timer, ptrs, n, None, steps, 5)
            stamps = torch.zeros(4 * grid, dtype=torch.int64, device="cuda")
            acc = np.zeros(5)
            reps = 20
            done = np.zeros(grid)
            for r in range(reps):
                stamps.zero_()
                B.mfr_sum_f16_stamped(ptrs[(r + 7) % len(ptrs)], n, timer.out.data_ptr(), None, stamps.data_ptr(), 4 * grid, timer.stream)
                torch.cuda.synchronize()
                st = stamps.cpu().numpy().reshape(grid, 4).astype(np.float64)
                t0 = st[:, 0].min()
                stored = st[:, 3].max()
                acc += np.array([st[:, 0].max() - t0, st[:, 1].min() - t0, st[:, 1].max() - t0, st[:, 2].max() - t0, stored - t0]) * tick_us
                done += (st[:, 1] - t0) * tick_us
            acc /= reps
            done /= reps
            if k in (26, 28):
                by_xcd = [done[np.arange(grid) % 8 == j].mean() for j in range(8)]
                notes.append("# n = 2^%d: mean time at which a block is done with its chains %.2f; by block index mod 8 (blocks are dealt to the "
                             "eight XCDs in turn): %s; slowest and fastest block on average %.2f / %.2f"
                             % (k, done.mean(), " ".join("%.2f" % v for v in by_xcd), done.max(), done.min()))
            emit(f, "%d %d %.2f %.2f %.2f %.2f %.2f %.2f %.2f" % (n, grid, period * 1e6, acc[0], acc[1], acc[2], acc[3], acc[4], 2 * n / 8e6))
        for line in notes:
            emit(f, line)


def run(args):
    import numpy as np
    import torch
    from paper_2001_05585_amd import binding as B
    from paper_2001_05585_amd import workloads as W
    if not torch.cuda.is_available():
        raise SystemExit("sweeps need a GPU")
    torch.cuda.set_device(0)
    B.lib()
    {"config2": config2, "config5": config5, "types": types, "rows": rows, "row_lengths": row_lengths, "split": split, "variants": variants, "wide": wide, "timeline": timeline}[args.sweep](args, torch, np, B, W)
