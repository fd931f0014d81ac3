"""Host logic of the many-rows kernel, checked without a GPU.

``mfr_rows_plan`` returns the shape the library would launch; the kernel's
index arithmetic (documented with that call) is replayed here per lane, and the
test checks what the kernel relies on for memory safety and for correctness:

* every element of every row is kept by exactly one (step, tile, lane),
* the slots of unmasked steps lie wholly inside their row,
* every load of the masked last step (including the substitute slot of a lane
  past the row's end) lies inside the array's span, for the rows the kernel is
  given; the rows it is not given are few,
* rows map to store lanes one to one,
* where the rows end in tail tiles, the tiles' slots cover exactly what the plain steps leave, their loads stay
  inside the span, and each storing lane fetches the tile and column that hold its own row,
* where rows of a 16-bit type at odd element addresses are read from one element earlier, every load starts on a
  4-byte boundary, none starts below the aligned word that holds x[0], and the element before the row is dropped.
"""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from paper_2001_05585_amd import binding as B

ESIZE = {B.MFR_DTYPE_F16: 2, B.MFR_DTYPE_BF16: 2, B.MFR_DTYPE_F32: 4}


def replay(x_addr, dtype, rows, cols, stride, cus=256):
    plan = B.mfr_rows_plan(x_addr, dtype, rows, cols, stride, cus)
    if plan is None:
        return None
    P, D, GF, iters, batches, plain_lo, plain_hi, row_lo, row_hi, all_plain, grid, flags = plan
    tail, shift, PT = flags & 1, (flags >> 1) & 1, 1 << (flags >> 2)        # PT: columns per row in a tail tile
    es = ESIZE[dtype]
    E = 16 // es
    RPT = 16 // P
    rpi = GF * RPT
    assert iters == -(-rows // rpi)
    assert 1 <= grid <= 2 * cus and grid * 4 >= min(iters, cus * 4) - 3          # one block per CU, some shapes two
    span = ((rows - 1) * stride + cols) * es
    lane = np.arange(64)
    j, q = lane & 15, lane >> 4
    part, row_local = j & (P - 1), j // P
    s_lane = part + P * q
    covered = np.zeros((rows, cols), dtype=np.int32)
    stored = np.zeros(rows, dtype=np.int32)
    assert plain_lo == 0 and row_lo == 0
    assert batches - 1 <= plain_hi <= batches          # at most the last step is masked
    if shift:
        assert es == 2 and D == 1 and (tail or not all_plain)
        assert (x_addr & 2) or ((stride * es) & 2)       # some row does start at an odd element address
    if tail:
        assert all_plain == 1 and D == 1 and batches >= 1 and PT in (1, 2, 4)
        rest = cols + shift - batches * 4 * P * E        # elements after the plain steps
        assert 0 < rest <= 4 * PT * E
        rptt = 16 // PT                                  # rows per tail tile
        ntt = -(-rpi * PT // 16)                         # tail tiles per iteration: one (maybe not full), or all full
        assert ntt == 1 or rpi * PT == ntt * 16
    else:
        assert PT == 1

    def odd_start(off):                                  # rows read from one element earlier
        return ((x_addr + off) >> 1) & 1 if shift else np.zeros_like(off)

    def check_loads(addr, odd):                          # byte offsets from x of 16-byte loads
        assert np.all(addr + x_addr >= (x_addr & ~3)) and np.all(addr + 16 <= span)
        if shift:
            assert np.all((addr + x_addr) % 4 == 0)
        else:
            assert np.all(addr >= 0)
    assert all_plain == (1 if plain_hi == batches else 0)
    if all_plain and not tail:
        assert row_hi == rows
    assert 0 < row_hi <= rows and rows - row_hi <= 8    # only rows within 16 bytes of the end are left out
    for it in range(iters):
        for u in range(GF):
            r_raw = (it * GF + u) * RPT + row_local
            r = np.minimum(r_raw, row_hi - 1)
            off = r * stride * es                  # byte offset of the row's first element from x
            odd = odd_start(off)
            base = off - 2 * odd                   # where the row's slots are counted from
            for cb in range(batches):
                plain = cb < plain_hi
                for d in range(D):
                    s = s_lane + 4 * P * (d + D * cb)
                    rel = base + 16 * s
                    e0 = E * s - odd               # column of the slot's first element (-1: the element before the row)
                    lo = np.where(e0 < 0, 1, 0)    # dropped from the first slot of a shifted row
                    if plain:
                        # the slot must be whole and inside the row
                        assert np.all(e0 + E <= cols), (it, u, cb, d)
                        check_loads(rel, odd)
                        hi = np.full(64, E)
                    else:
                        hi = np.clip(cols - e0, 0, E)
                        hi_loaded = np.clip(cols + shift - E * s, 0, E)     # the kernel decides on the longer, shifted row
                        addr = np.where(hi_loaded > 0, rel, base)           # a slot past the end is replaced by the first slot
                        check_loads(addr, odd)
                    for ln in range(64):
                        if r_raw[ln] >= row_hi:
                            continue
                        for t in range(lo[ln], hi[ln]):
                            c = e0[ln] + t
                            assert 0 <= c < cols
                            covered[r[ln], c] += 1
            # store lanes: part 0, q == u mod 4
            mine = (part == 0) & (q == (u & 3)) & (r_raw < row_hi)
            for ln in np.nonzero(mine)[0]:
                stored[r_raw[ln]] += 1
                if tail:
                    # the tail tile and column this lane fetches its row's rest from
                    h = u // 4
                    row_i = (4 * h + q[ln]) * RPT + row_local[ln]
                    tile, column = row_i // rptt, (row_i % rptt) * PT
                    assert tile < ntt and it * rpi + tile * rptt + column // PT == r_raw[ln]
        if tail:
            # tail tile t: lane (q, j) reads slot 4 P batches + (j mod PT) + PT q of row j // PT of the tile
            row_t = j // PT
            in_tail = row_t < rpi
            for tile in range(ntt):
                r_raw = it * rpi + tile * rptt + np.where(in_tail, row_t, 0)
                r = np.minimum(r_raw, row_hi - 1)
                off = r * stride * es
                odd = odd_start(off)
                base = off - 2 * odd
                s = 4 * P * batches + (j & (PT - 1)) + PT * q
                e0 = E * s - odd
                hi = np.where(in_tail, np.clip(cols - e0, 0, E), 0)
                hi_loaded = np.where(in_tail, np.clip(cols + shift - E * s, 0, E), 0)
                addr = np.where(hi_loaded > 0, base + 16 * s, base)
                check_loads(addr, odd)
                for ln in range(64):
                    if not in_tail[ln] or r_raw[ln] >= row_hi:
                        continue
                    for t in range(hi[ln]):
                        covered[r[ln], e0[ln] + t] += 1
    assert np.all(covered[:row_hi] == 1) and not covered[row_hi:].any()
    assert np.all(stored[:row_hi] == 1) and not stored[row_hi:].any()
    return plan


SHAPES = [
    # (x_addr low bits, rows, cols, stride) -- many rows so that the tiled kernel is chosen
    (0, 2048, 64, 64), (0, 2048, 32, 32), (0, 2048, 128, 128), (0, 2048, 256, 256), (0, 2048, 512, 512),
    (0, 2048, 1024, 1024), (0, 2100, 100, 100), (2, 2049, 64, 64), (14, 2048, 64, 72), (6, 2048, 7, 7),
    (0, 2048, 1, 1), (2, 2048, 1, 1), (0, 2048, 3, 5), (8, 2500, 33, 40), (0, 2048, 1001, 1001),
    (4, 2048, 520, 523), (0, 600, 700, 704), (4, 600, 3000, 3002), (0, 600, 2304, 2312), (2, 1100, 2000, 2001),
    (0, 2048, 384, 384), (0, 2048, 640, 640), (0, 2048, 768, 768), (0, 2048, 300, 300), (6, 2048, 350, 353), (0, 2048, 700, 704),
    (0, 1040, 33, 37), (6, 1033, 3, 3),
    # whole steps and a few bytes: the tail tile
    (0, 2048, 257, 257), (0, 2048, 260, 260), (2, 1100, 514, 514), (0, 1030, 1030, 1030), (4, 1027, 515, 520),
    (0, 1100, 2052, 2052), (0, 1030, 544, 544), (0, 2048, 288, 288), (0, 2048, 289, 289), (0, 1100, 2056, 2056),
    # 16-bit rows 2 bytes off a 4-byte boundary (all of them, or every other one): read from one element earlier
    (2, 2048, 256, 256), (2, 2048, 128, 128), (6, 2048, 150, 150), (0, 2048, 129, 129), (2, 1100, 512, 512),
    (0, 1100, 1025, 1025), (2, 1030, 300, 300), (2, 2048, 16, 16), (0, 2048, 17, 17), (6, 700, 1000, 1001),
    (2, 2048, 159, 160), (0, 1040, 31, 33), (2, 1100, 1024, 1026), (0, 1100, 1055, 1055), (2, 1100, 1500, 1500),
    # rests of up to 128 and 256 bytes: tail tiles with two and four columns per row
    (0, 2048, 300, 300), (0, 2048, 350, 352), (0, 2048, 384, 384), (0, 1100, 600, 600), (0, 1100, 640, 648), (0, 1030, 1100, 1100),
    (0, 1030, 1150, 1150), (2, 2048, 310, 310), (2, 2048, 380, 380), (0, 1100, 575, 575), (2, 1100, 1130, 1130), (0, 1030, 1600, 1608),
    # four steps and tail tiles (rows of 4 to 5 KiB)
    (0, 1030, 2100, 2100), (0, 1030, 2170, 2176), (4, 1030, 2052, 2060),
]


@pytest.mark.parametrize("dtype", [B.MFR_DTYPE_F16, B.MFR_DTYPE_F32])
@pytest.mark.parametrize("shape", SHAPES)
def test_replay_of_listed_shapes(dtype, shape):
    low, rows, cols, stride = shape
    es = ESIZE[dtype]
    x_addr = (1 << 20) + (low // es) * es
    if cols * rows > 1_500_000:
        rows = max(2048 if rows >= 2048 else rows, 1_500_000 // cols // 16 * 16)
    plan = replay(x_addr, dtype, rows, cols, stride)
    assert plan is not None


def test_power_of_two_rows_are_unmasked_at_any_alignment():
    for cols, P in ((32, 1), (64, 2), (128, 4), (256, 8), (512, 16), (1024, 16), (4096, 16)):
        plan = B.mfr_rows_plan(1 << 20, B.MFR_DTYPE_F16, 4096, cols, cols, 256)
        assert plan is not None and plan[0] == P and plan[9] == 1, (cols, plan)
    # binary32: a slot holds four values
    plan = B.mfr_rows_plan(1 << 20, B.MFR_DTYPE_F32, 4096, 64, 64, 256)
    assert plan[0] == 4 and plan[9] == 1
    # slots are counted from each row's first element: the base address and the stride do not matter
    plan = B.mfr_rows_plan((1 << 20) + 4, B.MFR_DTYPE_F16, 4096, 64, 66, 256)
    assert plan[0] == 2 and plan[9] == 1 and plan[8] == 4096 and plan[11] == 0
    # ... unless rows of a 16-bit type start 2 bytes off a 4-byte boundary: read from that boundary, such a row
    # is one element longer, and with it every row's plan
    for x_addr, stride in (((1 << 20) + 6, 66), (1 << 20, 67)):
        plan = B.mfr_rows_plan(x_addr, B.MFR_DTYPE_F16, 4096, 64, stride, 256)
        assert plan[0] == 4 and plan[9] == 0 and plan[11] == 2
    plan = B.mfr_rows_plan((1 << 20) + 4, B.MFR_DTYPE_F32, 4096, 64, 65, 256)
    assert plan[9] == 1 and plan[11] == 0


def test_rows_over_512_bytes_take_the_shape_that_wastes_least():
    f16, f32 = B.MFR_DTYPE_F16, B.MFR_DTYPE_F32
    shape = lambda dt, cols: B.mfr_rows_plan(1 << 20, dt, 4096, cols, cols, 256)
    assert shape(f16, 384)[:3] == (4, 1, 4) and shape(f16, 384)[9] == 1      # 768 B = 3 whole steps of 256 B
    assert shape(f16, 640)[:3] == (4, 1, 4) and shape(f16, 640)[4] == 5
    assert shape(f16, 768)[:3] == (8, 1, 4) and shape(f16, 768)[9] == 1      # 1536 B = 3 whole steps of 512 B
    assert shape(f32, 192)[:3] == (4, 1, 4) and shape(f32, 384)[:3] == (8, 1, 4)
    assert shape(f16, 260)[:3] == (8, 1, 8) and shape(f16, 260)[4] == 1 and shape(f16, 260)[11] == 1   # 512 B + 8: tail tile
    assert shape(f16, 520)[:3] == (16, 1, 8) and shape(f16, 520)[4] == 1 and shape(f16, 520)[11] == 1  # 1024 B + 16
    assert shape(f16, 700)[:3] == (16, 1, 8) and shape(f16, 700)[4] == 2 and shape(f16, 700)[11] == 0  # 1400 B: a masked second step
    assert shape(f16, 544)[11] == 1 and shape(f16, 288)[11] == 1         # at most 64 bytes after the steps: one column per row
    assert shape(f16, 290)[11] == 1 | 1 << 2 and shape(f16, 320)[11] == 1 | 1 << 2      # 65 to 128 bytes: two columns per row
    assert shape(f16, 322)[11] == 1 | 2 << 2 and shape(f16, 382)[11] == 1 | 2 << 2      # 129 to 256 bytes: four
    assert shape(f16, 384)[11] == 0 and shape(f16, 386)[11] == 0                        # whole 256-byte steps; 260 bytes after a step
    assert shape(f16, 600)[:3] == (16, 1, 8) and shape(f16, 600)[4] == 1 and shape(f16, 600)[11] == 1 | 2 << 2   # 1024 B + 176
    assert shape(f16, 1150)[:3] == (16, 1, 4) and shape(f16, 1150)[4] == 2 and shape(f16, 1150)[11] == 1 | 2 << 2  # 2048 B + 252
    assert shape(f16, 1600)[11] == 1 | 1 << 2 and shape(f16, 1650)[11] == 1 | 2 << 2 and shape(f16, 1670)[11] == 0   # 3200, 3300, 3340 B
    # shifted rows: the element before the row counts (bit 1 of plan[11]); the tail tile (bit 0) from 256-byte rows on
    shifted = lambda cols: B.mfr_rows_plan((1 << 20) + 2, f16, 4096, cols, cols, 256)
    assert shifted(256)[:3] == (8, 1, 8) and shifted(256)[4] == 1 and shifted(256)[11] == 3
    assert shifted(128)[:3] == (4, 1, 4) and shifted(128)[4] == 1 and shifted(128)[11] == 3
    assert shifted(287)[11] == 3 and shifted(288)[11] == 3 | 1 << 2 and shape(f16, 287)[11] == 3 and shape(f16, 289)[11] == 3 | 1 << 2
    assert shifted(383)[11] == 3 | 2 << 2 and shifted(384)[11] == 2        # 768 + 2 bytes to hold: 258 after the step
    assert shifted(1024)[:3] == (16, 1, 4) and shifted(1024)[4] == 2 and shifted(1024)[11] == 3
    assert shifted(255)[:3] == (8, 1, 8) and shifted(255)[9] == 0 and shifted(255)[11] == 2      # 256 elements to hold: one masked step
    # a single masked step under 69 % full, and 256-byte steps with a tail tile: two blocks per CU
    many = lambda dt, cols, x_addr=1 << 20: B.mfr_rows_plan(x_addr, dt, 1 << 18, cols, cols, 256)
    assert many(f16, 165)[10] == 512 and many(f16, 16)[10] == 512 and many(f32, 40)[10] == 512
    assert many(f16, 128, (1 << 20) + 2)[10] == 512
    assert many(f16, 400)[10] == 256 and many(f16, 24)[10] == 256 and many(f16, 600)[10] == 256 and many(f16, 290)[10] == 256
    assert many(f16, 256, (1 << 20) + 2)[10] == 256
    # a masked row of P = 16: eight groups when one step, or when under 80 % of the steps is filled
    assert shape(f16, 390)[:3] == (16, 1, 8) and shape(f16, 400)[:3] == (16, 1, 8) and shape(f16, 511)[:3] == (16, 1, 8)
    assert shape(f16, 800)[:3] == (16, 1, 8) and shape(f16, 800)[11] == 0 and shape(f16, 1200)[:3] == (16, 1, 8)
    assert shape(f16, 900)[:3] == (16, 1, 4) and shape(f16, 1000)[:3] == (16, 1, 4) and shape(f16, 2000)[:3] == (16, 1, 4)
    assert shape(f16, 1030)[:3] == (16, 1, 4) and shape(f16, 1030)[11] == 1   # 2048 B + 12: P = 16, two plain steps, tail tile
    assert shape(f16, 2052)[:3] == (16, 1, 4) and shape(f16, 2052)[4] == 4 and shape(f16, 2052)[11] == 1     # 4096 B + 8
    assert shape(f16, 2564)[11] == 0                                          # from 5 KiB on: no tail tiles
    assert shape(f16, 1200)[11] == 0
    assert shape(f16, 512)[:3] == (16, 1, 4) and shape(f16, 1024)[:3] == (16, 1, 4) and shape(f16, 1536)[:3] == (16, 1, 4)


def test_choice_between_kernels():
    f16 = B.MFR_DTYPE_F16
    assert B.mfr_rows_plan(1 << 20, f16, 1, 1000, 1000, 256) is None          # one row: the single-sum path
    assert B.mfr_rows_plan(1 << 20, f16, 100, 1 << 20, 1 << 20, 256) is None   # few long rows: a grid per row
    assert B.mfr_rows_plan(1 << 20, f16, 100, 64, 64, 256) is None
    assert B.mfr_rows_plan(1 << 20, f16, 100, 1001, 1001, 256) is None         # ... whatever their phases
    assert B.mfr_rows_plan(1 << 20, f16, 600, 4096, 4096, 256) is not None     # long rows from 512 rows on
    assert B.mfr_rows_plan(1 << 20, f16, 600, 4098, 4098, 256) is not None
    assert B.mfr_rows_plan(1 << 20, f16, 4096, 8, 8, 256) is not None
    assert B.mfr_rows_plan(1 << 20, f16, 4096, 8191, 8192, 256) is not None
    assert B.mfr_rows_plan(1 << 20, f16, 4096, 8192, 8192, 256) is None        # rows from 16 KiB on: a grid per row
    assert B.mfr_rows_plan(1 << 20, f16, 4096, 16385, 16385, 256) is None
    # 16-bit rows of 4 KiB or more that start 2 bytes off a 4-byte boundary: a grid per row (aligned slots)
    assert B.mfr_rows_plan(1 << 20, f16, 600, 4097, 4097, 256) is None
    assert B.mfr_rows_plan((1 << 20) + 2, f16, 600, 4096, 4096, 256) is None
    assert B.mfr_rows_plan((1 << 20) + 4, f16, 600, 4096, 4096, 256) is not None
    assert B.mfr_rows_plan((1 << 20) + 2, f16, 4096, 2047, 2047, 256) is not None
    assert B.mfr_rows_plan((1 << 20) + 4, B.MFR_DTYPE_F32, 600, 2049, 2049, 256) is not None
    # long rows: four tiles of one row per step, unless that wastes over a fifth of the steps
    assert B.mfr_rows_plan(1 << 20, f16, 600, 6000, 6000, 256)[:3] == (16, 4, 1)
    assert B.mfr_rows_plan(1 << 20, f16, 600, 2304, 2304, 256)[:3] == (16, 1, 4)
    assert B.mfr_rows_plan(1 << 20, f16, 600, 2560, 2560, 256)[:3] == (16, 4, 1)     # stride a multiple of 1 KiB


def test_invalid_arguments():
    plan = (B.ctypes.c_ulonglong * 12)()
    L = B.lib()
    assert L.mfr_rows_plan(1 << 20, 9, 4096, 64, 64, 256, plan) == -B.MFR_ERR_INVALID_ARG
    assert L.mfr_rows_plan((1 << 20) + 1, B.MFR_DTYPE_F16, 4096, 64, 64, 256, plan) == -B.MFR_ERR_INVALID_ARG
    assert L.mfr_rows_plan(1 << 20, B.MFR_DTYPE_F16, 4096, 64, 63, 256, plan) == -B.MFR_ERR_INVALID_ARG
    assert L.mfr_rows_plan(1 << 20, B.MFR_DTYPE_F16, 4096, 64, 64, 0, plan) == -B.MFR_ERR_INVALID_ARG
    assert L.mfr_rows_plan(1 << 20, B.MFR_DTYPE_F16, 4096, 64, 64, 256, None) == -B.MFR_ERR_INVALID_ARG
    assert L.mfr_rows_plan(1 << 20, B.MFR_DTYPE_F16, 4096, 64, 1 << 50, 256, plan) == -B.MFR_ERR_INVALID_ARG   # span wraps
    assert L.mfr_rows_plan(1 << 20, B.MFR_DTYPE_F16, 4096, 64, 1 << 40, 256, plan) == 1


@settings(max_examples=60, deadline=None)
@given(dtype=st.sampled_from([B.MFR_DTYPE_F16, B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32]),
       low=st.integers(0, 7), rows=st.integers(512, 2300), cols=st.integers(1, 300), gap=st.integers(0, 9),
       cus=st.sampled_from([1, 8, 256]))
def test_replay_of_random_shapes(dtype, low, rows, cols, gap, cus):
    es = ESIZE[dtype]
    x_addr = (1 << 20) + (low * 2 // es) * es
    if rows * cols > 200_000:
        cols = max(1, 200_000 // rows)
    replay(x_addr, dtype, rows, cols, cols + gap, cus)


@settings(max_examples=25, deadline=None)
@given(dtype=st.sampled_from([B.MFR_DTYPE_F16, B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32]),
       low=st.integers(0, 7), rows=st.integers(1024, 1060), cols=st.integers(129, 2600), gap=st.integers(0, 9))
def test_replay_of_random_longer_rows(dtype, low, rows, cols, gap):
    """Rows of several steps: tail tiles of every width after one to three steps, masked and shifted steps."""
    es = ESIZE[dtype]
    x_addr = (1 << 20) + (low * 2 // es) * es
    replay(x_addr, dtype, rows, cols, cols + gap, 256)

