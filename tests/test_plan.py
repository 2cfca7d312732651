"""Host logic without a GPU: how the many-rows GEMM cuts its work (the rule the kernels
evaluate on the device, through its inspection entry point).  The expected values are worked
out by hand from the rule as the header states it: a work item is 256 features wide and 256,
192 or 128 rows tall and moves 2 x (8 + 2 rt) KiB of operands per 32-k step (rt = rows / 64);
with K in S > 1 parts it also moves 256 rt KiB for its partial rows (64 rt rows x 256 features
x 4 bytes, written once, read once, counted twice); the estimate is rounds of 256 items x the
KiB of an item; ties go to the taller item and the fewer parts."""
import ctypes as C

import pytest

import paper_2502_02175_amd as V

PLAN = V.vlac_plan_many_rows_gemm


def test_large_launches_are_not_split():
    # 7B gate/up at 2712 rows: 86 tiles; 256-row items: 11 blocks, 946 items, 4 rounds x 4096 KiB;
    # 192-row: 15 blocks, 1290 items, 6 rounds x 3584; 128-row: 22 blocks, 8 rounds x 3072
    assert PLAN(2 * 11008, 4096, 2712, 1) == (256, 1, 946)
    # 7B QKV at 2712 rows: 48 tiles; 528 items of 256 rows take 3 rounds x 4096, 720 items of 192
    # rows 3 rounds x 3584, 1056 items of 128 rows 5 rounds x 3072
    assert PLAN(12288, 4096, 2712, 1) == (192, 1, 720)
    # 4096-wide projection with K 11008 (344 steps) at 8448 rows, residual epilogue: 704 items of
    # 192 rows in 3 rounds x 9632 KiB; two parts would take 5 rounds x 6528
    assert PLAN(4096, 11008, 8448, 3) == (192, 1, 704)


def test_few_items_are_cut_finer():
    # d_model 1536 (6 tiles), K 8960 (280 steps), 3584 rows: 84 items of 256 rows leave two
    # thirds of the CUs idle; 3 parts of 94 steps: 252 items x (3008 + 1024) KiB in one round
    assert PLAN(1536, 8960, 3584, 3) == (256, 3, 252)
    # the same without a residual epilogue: the shortest items (168 x 6720 KiB, one round)
    assert PLAN(1536, 8960, 3584, 1) == (128, 1, 168)
    # K 1536 (48 steps): the partial rows of a split would outweigh the operands
    assert PLAN(1536, 1536, 3584, 3) == (128, 1, 168)
    # 4096-wide projection, K 4096 (128 steps), 664 rows: 3 parts x 4 blocks of 192 rows x 16 tiles
    # = 192 items x (1204 + 768) KiB against 96 unsplit items of 128 rows x 3072 KiB
    assert PLAN(4096, 4096, 664, 3) == (192, 3, 192)
    # K below 1536 carries no split at all
    assert PLAN(1536, 1024, 3584, 3) == (128, 1, 168)


def test_up_to_eight_parts_where_the_workspace_allows():
    # the parts tried are 1, 2, 3, 4, 6 and 8.  4096 x 4096 at 446 rows: 4 blocks of 128 rows x
    # 16 tiles x 4 parts = 256 items x (24 x 32 + 512) = 1280 KiB in one round; 3 parts: 192
    # items x 1544; 8 parts of 256-row items: 256 items x (32 x 16 + 1024) = 1536
    assert PLAN(4096, 4096, 446, 8) == (128, 4, 256)
    # 4096 x 11008 (344 steps) at 344 rows: 2 blocks of 192 rows x 16 tiles x 8 parts = 256 items
    # x (28 x 43 + 768) = 1972 KiB; 256-row items in 8 parts: 32 x 43 + 1024 = 2400; 128-row
    # items: 3 blocks, 4 parts, 192 items x (24 x 86 + 512) = 2576
    assert PLAN(4096, 11008, 344, 8) == (192, 8, 256)
    # a limit of 5 admits 1, 2, 3 and 4
    assert PLAN(4096, 11008, 344, 5) == (128, 4, 192)


@pytest.mark.parametrize("n", [1536, 2048, 4096, 12288, 17920, 22016])
@pytest.mark.parametrize("k", [1024, 1536, 4096, 8960, 11008])
@pytest.mark.parametrize("smax", [1, 3, 8])
def test_invariants_over_row_counts(n, k, smax):
    tiles = -(-n // 256)
    for rows in list(range(1, 700, 37)) + list(range(700, 9000, 411)):
        block, s, items = PLAN(n, k, rows, smax)
        assert block in (128, 192, 256) and 1 <= s <= smax
        assert items == tiles * s * -(-rows // block)
        if s > 1:
            assert k >= 1536
        # never more rounds of 256 items than the plainest cut (256-row items, unsplit) would take
        # at a higher cost per item: the chosen estimate is the least of those tried
        steps = lambda S: -(-2 * (-(-k // 64)) // S)
        cost = lambda b, S: -(-(tiles * S * -(-rows // b)) // 256) * (2 * (8 + b // 32) * steps(S) + (4 * b if S > 1 else 0))
        assert cost(block, s) == min(cost(b, S) for b in (128, 192, 256) for S in (1, 2, 3, 4, 6, 8) if S <= (smax if k >= 1536 else 1))


def test_bad_arguments():
    lib = V.lib()
    out = C.c_int()
    assert lib.vlac_plan_many_rows_gemm(4096, 4096, 100, 1, None, C.byref(out), C.byref(out)) == -1
    for bad in ((0, 4096, 100, 1), (4096, 0, 100, 1), (4096, 4096, 0, 1), (4096, 4096, 100, 0)):
        assert lib.vlac_plan_many_rows_gemm(*bad, C.byref(out), C.byref(out), C.byref(out)) == -3
