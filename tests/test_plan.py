"""Host logic without a GPU: how the many-rows GEMM cuts its work (the rule the kernels
evaluate on the device, through its inspection entry point)."""
import ctypes as C

import pytest

import paper_2502_02175_amd as V

PLAN = V.vlac_plan_many_rows_gemm


def test_large_launches_keep_the_wide_unsplit_tile():
    # 7B gate/up at 2712 rows: 43 wide tiles x 22 row blocks, several rounds of 256 items
    assert PLAN(2 * 11008, 4096, 2712, 1) == (512, 1, 43 * 22)
    # 4096-wide projection at 8448 rows, residual epilogue: no split either
    assert PLAN(4096, 11008, 8448, 3) == (512, 1, 8 * 66)


def test_few_items_are_cut_finer_but_fit_one_round():
    # d_model 1536 (3 wide tiles), K 8960, 3584 rows (28 blocks): 84 items -> 3 K splits of the wide tile
    assert PLAN(1536, 8960, 3584, 3) == (512, 3, 252)
    # the same without a residual epilogue: narrow tiles only
    assert PLAN(1536, 8960, 3584, 1) == (256, 1, 168)
    # 4096-wide projection at 664 rows (6 blocks): 48 items -> narrow tiles in 2 splits
    assert PLAN(4096, 4096, 664, 3) == (256, 2, 192)
    # short K carries no split
    assert PLAN(1536, 1536, 3584, 3) == (256, 1, 168)


def test_a_little_more_than_a_round_takes_the_narrow_tile():
    # 8 wide tiles x 34 row blocks = 272 items (two rounds) -> 544 narrow ones (three shorter rounds)
    assert PLAN(4096, 4096, 4352, 3) == (256, 1, 544)
    # 24 wide tiles x 22 blocks = 528 items: three rounds either way, stays wide
    assert PLAN(12288, 4096, 2712, 1) == (512, 1, 528)


@pytest.mark.parametrize("n", [1536, 2048, 4096, 12288, 17920, 22016])
@pytest.mark.parametrize("k", [1536, 4096, 8960, 11008])
@pytest.mark.parametrize("smax", [1, 3])
def test_invariants_over_row_counts(n, k, smax):
    prev_items_per_block = None
    for rows in list(range(1, 700, 37)) + list(range(700, 9000, 411)):
        tile, s, items = PLAN(n, k, rows, smax)
        blocks = (rows + 127) // 128
        tiles = -(-n // tile)
        assert tile in (256, 512) and 1 <= s <= smax
        assert items == tiles * s * blocks
        if s > 1:
            assert k >= 4096 and items <= 256          # splits only for long K, and only within one round
        wide_items = -(-n // 512) * blocks
        if wide_items > 128 and wide_items <= 256:
            assert (tile, s) == (512, 1)                # no finer cut fits one round
        if tile == 256 and wide_items <= 256:
            assert items <= 256


def test_bad_arguments():
    lib = V.lib()
    out = C.c_int()
    assert lib.vlac_plan_many_rows_gemm(4096, 4096, 100, 1, None, C.byref(out), C.byref(out)) == -1
    for bad in ((0, 4096, 100, 1), (4096, 0, 100, 1), (4096, 4096, 0, 1), (4096, 4096, 100, 0)):
        assert lib.vlac_plan_many_rows_gemm(*bad, C.byref(out), C.byref(out), C.byref(out)) == -3
