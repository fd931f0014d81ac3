"""Host-side checks of the C-ABI boundary: run without a GPU.

The library must load, export every function ``include/mfreduce.h`` declares,
reject bad arguments before touching HIP, and split any (n, alignment,
geometry) so that every element is read exactly once and the unchecked 128-bit
loads stay inside [x, x + n).
"""
import ctypes
import os
import re

import pytest

from paper_2001_05585_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mfreduce.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mfr_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert "mfr_sum_f16" in names and "mfr_sum_f16_tuned" in names
    L = B.lib()
    for name in names:
        assert hasattr(L, name), name
    assert set(names) == set(B.EXPORTS)


def test_header_is_plain_c_and_the_library_links(tmp_path):
    import subprocess
    exe = str(tmp_path / "c_abi_check")
    src = os.path.join(ROOT, "tests", "c_abi_check.c")
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    src, "-o", exe, "-L", libdir, "-lmfreduce", "-Wl,-rpath," + libdir,
                    "-Wl,-rpath-link,/opt/rocm/lib"], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True)
    assert "c abi ok" in out.stdout


def test_version_and_strings():
    assert B.mfr_version() >= 100
    assert B.mfr_strerror(B.MFR_OK) == "success"
    for st in (B.MFR_ERR_INVALID_ARG, B.MFR_ERR_UNSUPPORTED, B.MFR_ERR_HIP, 77):
        assert B.mfr_strerror(st)
    b, r, g = B.mfr_get_default_tuning()
    assert b in (64, 128, 256, 512, 1024) and 1 <= r <= 8 and g == B.MFR_GRID_AUTO
    assert B.lib().mfr_get_default_tuning(None, None, None) == B.MFR_OK


def test_invalid_arguments_are_rejected_before_any_hip_call():
    L = B.lib()
    INV = B.MFR_ERR_INVALID_ARG
    assert L.mfr_sum_f16(None, 5, 4096, None) == INV          # null x, n > 0
    assert L.mfr_sum_f16(4096, 5, None, None) == INV          # null out
    assert L.mfr_sum_f16(None, 0, None, None) == INV          # null out even when n == 0
    assert L.mfr_sum_f16(4097, 5, 4096, None) == INV          # x not 2-byte aligned
    assert L.mfr_sum_f16(4096, (1 << 60) + 1, 4096, None) == INV
    for block in (0, 1, 16, 48, 96, 2048, -64):
        assert L.mfr_sum_f16_tuned(4096, 5, 4096, block, 1, 0, 0, None) == INV
    for R in (0, -1, 9, 100):
        assert L.mfr_sum_f16_tuned(4096, 5, 4096, 256, R, 0, 0, None) == INV
    assert L.mfr_sum_f16_tuned(4096, 5, 4096, 256, 1, -2, 0, None) == INV
    assert L.mfr_sum_f16_tuned(4096, 5, 4096, 256, 1, 0, 3, None) == INV
    for kw in (dict(chains_in_flight=5), dict(chains_in_flight=7), dict(chains_in_flight=16), dict(chain_R=3, chains_in_flight=6), dict(chain_R=8, chains_in_flight=4),
               dict(nontemporal=3), dict(kernel=-1), dict(block_threads=100), dict(combine=3), dict(combine=-1),
               dict(kernel=2, split_permille=1001), dict(kernel=2, split_permille=-1), dict(kernel=0, split_permille=500),
               dict(kernel=2, block_threads=32)):
        t = B.make_tuning(**kw)
        assert L.mfr_sum_f16_ex(4096, 5, 4096, ctypes.byref(t), None) == INV
    with pytest.raises(B.MfrError):
        B.mfr_sum_f16(0, 5, 4096)


def simulate_coverage(n, x_addr, t, dtype=0):
    head, slots, main0, chains, ts, epi0, epi1 = B.mfr_plan_ex(n, x_addr, dtype, t)
    if dtype == 0:
        assert (head, slots, main0, chains, ts, epi0, epi1) == B.mfr_plan_for(n, x_addr, t)
    esize = 4 if dtype == B.MFR_DTYPE_F32 else 2
    per_slot = 16 // esize
    R = t.chain_R
    vend = head + n
    assert head == (x_addr % 16) // esize
    assert slots == -(-vend // per_slot)
    count = [0] * slots
    main_end = main0 + chains * R * ts
    for q in range(main0, main_end):
        assert per_slot * q >= head and per_slot * (q + 1) <= vend, "unchecked load outside [x, x+n)"
        count[q] += 1
    assert epi0 <= epi1
    assert epi1 - epi0 <= (R + 1) * ts, "border must fit in two masked chains"
    for p in range(epi0, epi1):
        q = p if p < slots else 0
        count[q] += 1
    assert all(c == 1 for c in count), (n, x_addr, t.block_threads, R)


@pytest.mark.parametrize("block", [32, 64, 256])
@pytest.mark.parametrize("R", [1, 3, 8])
def test_every_slot_is_covered_exactly_once(block, R):
    t = B.make_tuning(block, R)
    ts = 32 if block == 32 else 64
    edge = 8 * ts * R
    ns = set(range(1, 40)) | {edge + d for d in range(-9, 10)} | {3 * edge + d for d in range(-9, 10)}
    ns |= {511, 512, 513, 2047, 2048, 2049, 65536 + 7, 100003}
    for n in sorted(v for v in ns if v >= 1):
        for shift in range(8):
            simulate_coverage(n, 4096 + 2 * shift, t)


@pytest.mark.parametrize("dtype", [B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32])
def test_every_slot_is_covered_exactly_once_other_types(dtype):
    esize = 4 if dtype == B.MFR_DTYPE_F32 else 2
    for R in (1, 4):
        t = B.make_tuning(256, R)
        edge = (16 // esize) * 64 * R
        ns = set(range(1, 20)) | {edge + d for d in range(-5, 6)} | {2 * edge + d for d in range(-5, 6)} | {100003}
        for n in sorted(ns):
            for shift in range(16 // esize):
                simulate_coverage(n, 4096 + esize * shift, t, dtype)
    # the 32-thread geometry exists for binary16 only; unknown types are rejected
    plan = (ctypes.c_ulonglong * 7)()
    t32 = B.make_tuning(32, 1)
    assert B.lib().mfr_plan_ex(100, 4096, dtype, ctypes.byref(t32), plan) == B.MFR_ERR_INVALID_ARG
    assert B.lib().mfr_plan_ex(100, 4096, 7, None, plan) == B.MFR_ERR_INVALID_ARG


def test_typed_and_batched_entries_reject_bad_arguments():
    L = B.lib()
    INV = B.MFR_ERR_INVALID_ARG
    assert L.mfr_sum_f32(4098, 5, 4096, None) == INV             # not 4-byte aligned
    assert L.mfr_sum_bf16(4097, 5, 4096, None) == INV
    assert L.mfr_sum_ex(4096, 3, 5, 4096, None, None) == INV     # unknown element type
    assert L.mfr_sum_ex(4096, -1, 5, 4096, None, None) == INV
    assert L.mfr_sum_f32(None, 5, 4096, None) == INV
    assert L.mfr_sum_rows_ex(4096, 0, 4, 100, 99, 4096, None, None) == INV   # stride < cols
    assert L.mfr_sum_rows_ex(4096, 0, 4096, 100, 1 << 50, 4096, None, None) == INV   # span beyond 2^60 elements
    assert L.mfr_sum_rows_ex(None, 0, 4, 100, 100, 4096, None, None) == INV
    assert L.mfr_sum_rows_ex(4096, 0, 4, 100, 100, None, None, None) == INV
    assert L.mfr_sum_rows_ex(4096, 0, 0, 100, 100, 4096, None, None) == B.MFR_OK   # no rows: nothing to do
    assert L.mfr_sum_f16_rows(4097, 2, 8, 8, 4096, None) == INV
    split = B.make_tuning(kernel=B.MFR_KERNEL_SPLIT, split_permille=500)
    assert L.mfr_sum_ex(4096, B.MFR_DTYPE_F32, 5, 4096, ctypes.byref(split), None) == INV   # split: binary16 only


def test_grid_for_one_chain_geometry():
    # one chain per wave: ceil(chains / waves) blocks
    assert B.mfr_grid_for(1 << 28, 0, B.make_tuning(256, 1, -1)) == (1 << 28) // (512 * 4)
    assert B.mfr_grid_for(1 << 28, 0, B.make_tuning(128, 4, -1)) == (1 << 28) // (512 * 4 * 2)
    assert B.mfr_grid_for(1 << 20, 0, B.make_tuning(32, 1, -1)) == (1 << 20) // 256
    assert B.mfr_grid_for(100, 0, B.make_tuning(256, 1, -1)) == 1
    assert B.mfr_grid_for(0, 0, None) == 1
    assert B.mfr_grid_for(1 << 20, 0, B.make_tuning(256, 1, 7)) == 7
    assert B.mfr_grid_for(1 << 20, 0, B.make_tuning(100, 1, 7)) == -1


def _in_fresh_process(env, code):
    """Run `code` in a new interpreter (the library reads the environment once per process)."""
    import subprocess
    import sys
    full = dict(os.environ)
    full.update(env)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    return subprocess.run([sys.executable, "-c", code], env=full, cwd=root, capture_output=True, text=True, timeout=120)


def test_environment_override_of_the_default_geometry():
    code = ("from paper_2001_05585_amd import binding as B\n"
            "print(B.mfr_get_default_tuning())\n"
            "print(B.mfr_plan_for(1 << 20, 4096, None))\n")
    base = _in_fresh_process({"MFR_BLOCK": "", "MFR_R": ""}, "import os\nos.environ.pop('MFR_BLOCK'); os.environ.pop('MFR_R')\n" + code)
    assert base.returncode == 0, base.stderr
    assert base.stdout.splitlines()[0] == "(256, 3, 0)"
    r = _in_fresh_process({"MFR_BLOCK": "512", "MFR_R": "2"}, code)
    assert r.returncode == 0, r.stderr
    lines = r.stdout.splitlines()
    assert lines[0] == "(512, 2, 0)"
    # 2^20 halves = 2048 tiles of 64 slots: chains of R = 2 tiles instead of the 8 that an input of
    # 2 MiB gets by default (the override also switches the size-dependent defaults off)
    assert eval(lines[1])[3] == 1024 and eval(base.stdout.splitlines()[1])[3] == 256
    # explicit tuning is not affected
    r = _in_fresh_process({"MFR_BLOCK": "512", "MFR_R": "2"},
                          "from paper_2001_05585_amd import binding as B\n"
                          "print(B.mfr_plan_for(1 << 20, 4096, B.make_tuning(128, 8))[3])\n")
    assert r.stdout.strip() == "256"
    for bad in ({"MFR_BLOCK": "100"}, {"MFR_R": "9"}, {"MFR_R": "four"}, {"MFR_BLOCK": "256x"}):
        r = _in_fresh_process(bad, "from paper_2001_05585_amd import binding as B\n"
                                   "import ctypes\n"
                                   "b = ctypes.c_int()\n"
                                   "print(B.lib().mfr_get_default_tuning(ctypes.byref(b), None, None))\n"
                                   "plan = (ctypes.c_ulonglong * 7)()\n"
                                   "print(B.lib().mfr_plan_for(1 << 20, 4096, None, plan))\n"
                                   "print(B.lib().mfr_plan_for(1 << 20, 4096, ctypes.byref(B.make_tuning(128, 8)), plan))\n")
        assert r.returncode == 0, r.stderr
        assert r.stdout.split() == [str(B.MFR_ERR_INVALID_ARG), str(B.MFR_ERR_INVALID_ARG), str(B.MFR_OK)], (bad, r.stdout)
