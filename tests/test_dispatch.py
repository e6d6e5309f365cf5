"""Host logic: which kernels slope_spmm_fwd picks for a shape (slope_spmm_fwd_plan, no GPU needed).
The regimes pinned here are the ones the design notes describe; the boundaries are properties of the
cost estimates, not of measured times."""
import pytest

from paper_2405_16325_amd import binding as sl

STREAM, SLABS, TILE, GENERIC, STREAM_ROWS = 0, 1, 2, 3, 4


@pytest.mark.parametrize("b", [1, 7, 16, 17, 32])
@pytest.mark.parametrize("d_out,d_in", [(9216, 9216), (36864, 9216), (9216, 36864), (512, 128)])
def test_up_to_32_tokens_take_a_small_batch_kernel(b, d_out, d_in):
    p = sl.slope_spmm_fwd_plan(b, d_in, d_out)
    assert p["product"] in (STREAM, STREAM_ROWS)
    assert p["tokens"] == (16 if b <= 16 else 32)
    if p["product"] == STREAM:
        assert p["slabs"] == 1 and p["rows"] in ((32, 48, 64) if b <= 16 else (32, 48))
    else:
        assert p["rows"] == 48 and d_in % 1024 == 0 and p["slabs"] * -(-d_out // 48) >= 512


def test_row_split_form_of_the_small_batch_kernel():
    # a tall matrix: one workgroup per 48 rows fills the chip three times, no slices
    p = sl.slope_spmm_fwd_plan(16, 9216, 36864)
    assert (p["product"], p["slabs"]) == (STREAM_ROWS, 1)
    assert sl.slope_spmm_fwd_plan(16, 9216, 36864, 0, False)["product"] == STREAM_ROWS
    # 192 workgroups and a long contraction (36 chunks of 1024): cut into 4 slices with scratch, else the kernel
    # whose wavefronts split the contraction; 9 chunks are too few to pay for the second launch
    p = sl.slope_spmm_fwd_plan(16, 36864, 9216)
    assert (p["product"], p["slabs"]) == (STREAM_ROWS, 4)
    assert sl.slope_spmm_fwd_plan(16, 36864, 9216, 0, False)["product"] == STREAM
    assert sl.slope_spmm_fwd_plan(16, 9216, 9216)["product"] == STREAM
    # 17 to 32 tokens: only where a long contraction over few rows wants four slices or more
    assert sl.slope_spmm_fwd_plan(32, 36864, 9216)["product"] == STREAM_ROWS
    assert sl.slope_spmm_fwd_plan(32, 9216, 9216)["product"] == STREAM
    assert sl.slope_spmm_fwd_plan(32, 9216, 36864)["product"] == STREAM
    # 625 workgroups fill the chip without slices, which 9 chunks would not pay for: the same with and without scratch
    assert [sl.slope_spmm_fwd_plan(16, 9216, 30000, 0, ws)["slabs"] for ws in (True, False)] == [1, 1]
    assert sl.slope_spmm_fwd_plan(16, 9216, 30000)["product"] == STREAM_ROWS
    # contractions that are no multiple of 1024, and matrices too small to fill the chip either way
    assert sl.slope_spmm_fwd_plan(16, 2560, 36864)["product"] == STREAM
    assert sl.slope_spmm_fwd_plan(16, 1024, 2048)["product"] == STREAM


def test_small_batch_rows_avoid_a_thin_last_round():
    # 9216 rows: 288 workgroups of 32 rows would leave a last round of 32; 192 of 48 rows fit one round
    assert sl.slope_spmm_fwd_plan(1, 9216, 9216, 0, False)["rows"] == 48
    # 8192 rows: 256 workgroups of 32 rows are exactly one round
    assert sl.slope_spmm_fwd_plan(1, 9216, 8192, 0, False)["rows"] == 32


def test_contraction_shorter_than_two_k_steps_stays_off_the_small_batch_kernel():
    assert sl.slope_spmm_fwd_plan(4, 64, 512)["product"] != STREAM


@pytest.mark.parametrize("b", [33, 100, 128, 200, 256])
def test_mid_batches_split_the_contraction_only_with_scratch_and_few_tiles(b):
    with_ws = sl.slope_spmm_fwd_plan(b, 9216, 9216, 0, True)
    without = sl.slope_spmm_fwd_plan(b, 9216, 9216, 0, False)
    assert with_ws["product"] == SLABS and with_ws["slabs"] >= 2 and with_ws["rows"] == 256
    assert without["product"] == TILE and without["slabs"] == 1
    # 36864 weight rows and two token tiles: 288 tiles fill the chip, no split
    big = sl.slope_spmm_fwd_plan(b, 9216, 36864, 0, True)
    assert (big["product"] == SLABS) == (b <= 128)


def test_slabs_times_tiles_fits_one_round_for_two_token_tiles():
    p = sl.slope_spmm_fwd_plan(256, 9216, 9216, 0, True)       # 36 x 2 tiles
    assert p["slabs"] == 3                                      # 216 workgroups: one round; 4 slabs would need two


@pytest.mark.parametrize("b,d_out,d_in", [(16384, 9216, 9216), (16384, 36864, 9216), (16384, 9216, 36864)])
def test_large_training_shapes_take_the_largest_tile(b, d_out, d_in):
    p = sl.slope_spmm_fwd_plan(b, d_in, d_out, 0, True)
    assert p["product"] == TILE and (p["rows"], p["tokens"]) == (256, 256) and p["slabs"] == 1


def test_a_small_layer_gets_a_tile_that_fits_one_round():
    p = sl.slope_spmm_fwd_plan(2048, 768, 3072, 0, True)       # OPT-125m fc1
    tiles = -(-3072 // p["rows"]) * -(-2048 // p["tokens"])
    assert p["product"] == TILE and tiles <= 256


def test_contractions_that_are_no_multiple_of_256_take_the_generic_kernel():
    assert sl.slope_spmm_fwd_plan(300, 320, 448)["product"] == GENERIC
    assert sl.slope_spmm_fwd_plan(300, 512, 448)["product"] == TILE


def test_adapter_product_regimes():
    xl = lambda b, r=128, d_in=9216: sl.slope_spmm_fwd_plan(b, d_in, 9216, r)["xl"]
    assert sl.slope_spmm_fwd_plan(64, 9216, 9216, 0)["xl"] == 0
    assert [xl(b) for b in (1, 16, 17, 128, 512)] == [1] * 5    # split over d_in, L as stored
    assert [xl(b) for b in (513, 4096)] == [3, 3]               # dense tile kernel, too few tiles: split over d_in
    assert xl(16384) == 2                                       # 256 tiles: no split
    # chunks of 64 rows of L per workgroup: as many as still give every compute unit a workgroup
    chunks = lambda b, d_in: sl.slope_spmm_fwd_plan(b, d_in, 9216, 128)["xl_chunks"]
    assert chunks(16, 9216) == 1 and chunks(64, 9216) == 1 and chunks(16, 36864) == 2 and chunks(512, 36864) == 4


def test_plan_rejects_what_the_call_rejects():
    with pytest.raises(sl.SlopeError):
        sl.slope_spmm_fwd_plan(0, 9216, 9216)
    with pytest.raises(sl.SlopeError):
        sl.slope_spmm_fwd_plan(16, 9216, 9216, 48)
    with pytest.raises(sl.SlopeError):
        sl.slope_spmm_fwd_plan(16, 9204, 9216)


def test_extents_that_are_not_multiples_of_64_take_the_general_kernels():
    # any multiple of 8 is accepted; a contraction that is not a whole number of k-steps of 64 goes to the
    # generic kernel's form for ragged rows (also for inference-size batches) and to plain arithmetic for X L
    for b in (1, 16, 300, 5000):
        plan = sl.slope_spmm_fwd_plan(b, 1000, 1000, 64)
        assert plan["product"] == GENERIC and plan["xl"] == 4
    assert sl.slope_spmm_fwd_plan(16, 1024, 1000, 64)["product"] == 0      # d_out may be ragged on the fast paths
    assert sl.slope_spmm_fwd_plan(4096, 1024, 1000, 64)["product"] == TILE
