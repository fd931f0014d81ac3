"""Host logic of the per-row kernels of the batched form: block size, blocks per row, chain shape, stagger and
residency limit, as mfr_rows_geometry reports them (no GPU needed).

The rules are the library's own (measured choices, not the paper's); what is checked is that they hold together:
explicit tuning is passed through untouched, a device of 256 compute units is kept supplied with about one wave of
6 KiB of loads per SIMD whatever the row count, the stagger puts the rows on a 1 MiB lattice, and the boundaries
between the regimes are where the header and the measurements put them."""
import numpy as np
import pytest

from paper_2001_05585_amd import binding as B

F16, BF16, F32 = B.MFR_DTYPE_F16, B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32
CUS = 256
SIMDS = 4 * CUS
TARGET_TILES = 6 * SIMDS            # one wave per SIMD with six 1 KiB tiles in flight
MIB = 1 << 20


def esize(dtype):
    return 4 if dtype == F32 else 2


def long_rows(dtype, rows, total_bytes=1 << 29):
    """cols of `rows` contiguous rows filling total_bytes, whole 16-byte slots."""
    return total_bytes // esize(dtype) // rows // 8 * 8


def geometry(dtype, rows, cols, stride=None, t=None, x_addr=0x10000):
    return B.mfr_rows_geometry(x_addr, dtype, rows, cols, cols if stride is None else stride, t, CUS)


def test_symbol_and_argument_checks():
    B.lib()
    with pytest.raises(B.MfrError):
        geometry(F16, 0, 100)
    with pytest.raises(B.MfrError):
        geometry(F16, 4, 0)
    with pytest.raises(B.MfrError):
        geometry(F16, 4, 100, stride=99)
    with pytest.raises(B.MfrError):
        geometry(F32, 4, 100, x_addr=0x10002)
    with pytest.raises(B.MfrError):
        B.mfr_rows_geometry(0x10000, 7, 4, 100, 100, None, CUS)
    with pytest.raises(B.MfrError):
        B.mfr_rows_geometry(0x10000, F16, 4, 100, 100, None, 0)


def test_none_where_the_many_rows_kernel_takes_the_call():
    for dtype, rows, cols in ((F16, 1 << 16, 1024), (F32, 4096, 1000), (BF16, 1 << 20, 37)):
        assert B.mfr_rows_plan(0x10000, dtype, rows, cols, cols, CUS) is not None
        assert geometry(dtype, rows, cols) is None
        # explicit tuning always selects the per-row kernels
        assert geometry(dtype, rows, cols, t=B.make_tuning()) is not None


@pytest.mark.parametrize("dtype", [F16, F32])
def test_explicit_tuning_is_passed_through(dtype):
    for block, R, grid, U in ((64, 1, 1, 1), (256, 2, 3, 3), (128, 8, 7, 2), (1024, 4, 2, 4)):
        for rows, cols in ((2, 100000), (520, 66000), (1500, 70000), (70000, 3000)):
            g = geometry(dtype, rows, cols, t=B.make_tuning(block, R, grid, 0, U))
            assert g[:4] == (block, grid, R, U), (g, block, R, grid, U)
            assert g[5] == 0 and g[6] == 0, g            # neither stagger nor residency limit


@pytest.mark.parametrize("dtype", [F16, BF16, F32])
def test_every_row_count_keeps_the_device_supplied(dtype):
    """Rows that run side by side (fewer than four per CU, or a one-wave block per row): the waves of the launch
    together keep 0.8 to 2.1 times the target in flight, in chains of at most eight tiles."""
    for rows in range(2, 2048):
        g = geometry(dtype, rows, long_rows(dtype, rows))
        assert g is not None, rows
        block, per_row, R, U = g[:4]
        assert block in (64, 128, 256) and per_row >= 1 and 1 <= R <= 8 and U in (1, 2, 3, 4, 6, 8) and R * U <= 16, (rows, g)
        if rows >= SIMDS and block != 64:
            continue                                     # blocks in rounds, limited by plan[6]
        tiles = rows * per_row * (block // 64) * R * U
        assert 0.8 * TARGET_TILES <= tiles <= 2.1 * TARGET_TILES, (rows, g, tiles / TARGET_TILES)
        # never more waves than two per SIMD, never fewer than half the SIMDs busy from 128 rows on
        waves = rows * per_row * (block // 64)
        assert waves <= 2 * SIMDS + block // 64 * per_row, (rows, g)
        if rows >= 128:
            assert 2 * waves >= SIMDS, (rows, g)


def test_regime_boundaries():
    def g(dtype, rows, cols=None):
        return geometry(dtype, rows, long_rows(dtype, rows) if cols is None else cols)
    # one 256-thread block per CU shared among few rows
    assert g(F16, 2)[:4] == (256, 128, 3, 2) and g(F16, 256)[:4] == (256, 1, 3, 2)
    # a few hundred rows: one-wave blocks, deeper chains as the waves become fewer
    assert g(F16, 300)[:4] == (64, 3, 4, 2) and g(F32, 300)[:4] == (64, 3, 8, 1)
    assert g(F16, 600)[:4] == (64, 1, 6, 2) and g(F16, 700)[:4] == (64, 1, 6, 2)
    assert g(F16, 900)[:4] == (64, 1, 4, 2) and g(F32, 900)[:4] == (64, 1, 8, 1)
    assert g(F16, 1000)[:4] == (64, 1, 3, 2)
    assert g(F16, 512)[2] * g(F16, 512)[3] * (g(F16, 512)[0] // 64) * g(F16, 512)[1] == 12
    # a few rows more than half the SIMDs: two one-wave blocks with one chain of six tiles
    for dtype, last in ((F16, 544), (BF16, 544), (F32, 640)):
        assert g(dtype, 513)[:4] == (64, 2, 6, 1) and g(dtype, last)[:4] == (64, 2, 6, 1), dtype
        assert g(dtype, last + 1)[1] == 1, dtype
    assert g(F16, 520, cols=20000)[1] == 1               # rows under 64 KiB are not split
    # one to two rows per SIMD, rows of 64 KiB and more: a one-wave block per row, 6, 4 or 3 KiB in flight
    assert g(F16, 1024)[:4] == (64, 1, 3, 2) and g(F16, 1228)[:4] == (64, 1, 3, 2)
    assert g(F16, 1229)[:4] == (64, 1, 4, 1) and g(F16, 1660)[:4] == (64, 1, 4, 1)
    assert g(F16, 1661)[:4] == (64, 1, 3, 1) and g(F16, 2047)[:4] == (64, 1, 3, 1)
    assert g(F16, 2048)[0] == 256
    assert g(F32, 1663)[0] == 64 and g(F32, 1664)[0] == 256
    assert g(F16, 1500, cols=32768)[0] == 64 and g(F16, 1500, cols=32760)[0] == 256      # 64 KiB is the limit
    # more rows than that: the block size follows the row length
    assert geometry(F16, 4096, 8192, t=None)[0] == 128 and geometry(F16, 4096, 16384)[0] == 256
    assert geometry(F16, 4097, 5000, stride=5001)[0] == 64          # rows of differing phase, under 12 KiB


@pytest.mark.parametrize("dtype", [F16, F32])
def test_stagger_puts_the_rows_on_a_lattice_of_1_mib(dtype):
    rng = np.random.default_rng(5)
    es = esize(dtype)
    for _ in range(400):
        rows = int(rng.integers(2, 2048))
        cols = int(rng.integers(40000, 2_000_000))
        stride = cols + int(rng.choice([0, 0, 1, 8, 4096]))
        g = geometry(dtype, rows, cols, stride=stride)
        if g is None:
            continue
        pitch = stride * es
        side_by_side = rows < SIMDS or (g[0] == 64 and g[1] == 1 and cols * es >= 65536 and rows < 2 * SIMDS)
        if g[5]:
            assert side_by_side and g[4] > 16, (rows, cols, g)
            assert 0 < g[5] < MIB and (pitch + g[5]) % MIB == 0, (rows, cols, stride, g)
        elif side_by_side and g[4] > 16:
            assert pitch % MIB == 0, (rows, cols, stride, g)
    # a pitch that is a multiple of 1 MiB needs none; a single row has none
    assert geometry(dtype, 100, MIB // es)[5] == 0
    assert geometry(dtype, 100, MIB // es - 8, stride=MIB // es)[5] == 0
    assert geometry(dtype, 1, 5_000_000)[5] == 0
    assert geometry(dtype, 100, (3 * MIB - 4096) // es)[5] == 4096
    # short rows (at most 16 chains) start where they are
    assert geometry(dtype, 100, 3 * 1024 * 16 // es)[5] == 0


def test_residency_limit_only_for_many_blocks_of_whole_slot_rows():
    # 16384 rows of 32 KiB: limited; one element more per row (ragged last slot) or a row off a boundary: not
    assert geometry(F16, 16384, 16384)[6] > 0
    assert geometry(F16, 16384, 16385, stride=16392)[6] == 0
    assert geometry(F16, 16384, 16384, x_addr=0x10002)[6] == 0
    assert geometry(F16, 16384, 16384, t=B.make_tuning())[6] == 0
    # rows that run side by side are never limited
    for rows in (2, 300, 520, 1000, 1100, 2000):
        assert geometry(F16, rows, long_rows(F16, rows))[6] == 0, rows


def test_rows_of_differing_phase_are_flagged():
    assert geometry(F16, 300, 100003)[7] == 1
    assert geometry(F16, 300, 100003, stride=100008)[7] == 0
    assert geometry(F32, 300, 100002)[7] == 1
    assert geometry(F16, 1, 100003)[7] == 0
