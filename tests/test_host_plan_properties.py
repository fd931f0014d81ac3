"""Property tests (hypothesis) of the host-side geometry: for any size, alignment,
element type, block size and chain length the input is covered exactly once, the
unchecked 128-bit loads stay inside [x, x + n), and the border fits two chains."""
from hypothesis import given, settings, strategies as st

from paper_2001_05585_amd import binding as B


def check(n, shift, dtype, block, R):
    esize = 4 if dtype == B.MFR_DTYPE_F32 else 2
    per_slot = 16 // esize
    t = B.make_tuning(block, R)
    head, slots, main0, chains, ts, epi0, epi1 = B.mfr_plan_ex(n, 1 << 20 | (shift * esize), dtype, t)
    vend = head + n
    assert head == shift and slots == -(-vend // per_slot)
    assert ts == (32 if block == 32 else 64)
    main_end = main0 + chains * R * ts
    # main region: whole slots strictly inside the valid range
    if chains:
        assert per_slot * main0 >= head and per_slot * main_end <= vend
    # border: [main_end, slots) plus slot 0 when it is partial, nothing else, at most two chains
    assert epi0 == min(main_end, epi1)
    assert epi1 == slots + (1 if head else 0)
    assert epi1 - epi0 <= (R + 1) * ts
    assert main0 == (1 if head else 0)
    covered = (main_end - main0) + (epi1 - epi0)
    assert covered == slots, (n, shift, dtype, block, R)


@settings(max_examples=400, deadline=None)
@given(n=st.one_of(st.integers(1, 5000), st.integers(1, 1 << 40)), shift=st.integers(0, 7),
       block=st.sampled_from([32, 64, 128, 256, 512, 1024]), R=st.integers(1, 8))
def test_plan_covers_every_slot_once_f16(n, shift, block, R):
    check(n, shift, B.MFR_DTYPE_F16, block, R)


@settings(max_examples=300, deadline=None)
@given(n=st.one_of(st.integers(1, 5000), st.integers(1, 1 << 40)), shift=st.integers(0, 7),
       dtype=st.sampled_from([B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32]),
       block=st.sampled_from([64, 128, 256, 512, 1024]), R=st.integers(1, 8))
def test_plan_covers_every_slot_once_other_types(n, shift, dtype, block, R):
    if dtype == B.MFR_DTYPE_F32:
        shift %= 4
    check(n, shift, dtype, block, R)


@settings(max_examples=200, deadline=None)
@given(n=st.integers(1, 1 << 40), block=st.sampled_from([32, 64, 128, 256, 512, 1024]), R=st.integers(1, 8),
       grid=st.sampled_from([-1, 1, 7, 300, 70000]))
def test_grid_for_is_consistent(n, block, R, grid):
    t = B.make_tuning(block, R, grid)
    g = B.mfr_grid_for(n, 0, t)
    waves = max(1, block // 64)
    tile = 256 if block == 32 else 512
    chains = n // (tile * R)
    if grid == -1:
        want = max(1, -(-chains // waves))
        assert g == want or (want > 0x7fffffff and g == -1)
    else:
        assert g == grid

