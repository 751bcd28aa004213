"""Host-side checks of the launch plan (tile variant, split of the last round):
no GPU needed, the planner falls back to 256 CUs when there is no device."""
import pytest

import paper_1611_08035_amd as xg

WS = None


def name(prec, v):
    return xg.xgemm_variant_name(prec, v)


@pytest.fixture(autouse=True)
def _auto():
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)
    yield
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)


def test_benchmark_configurations_fill_their_rounds_and_are_never_split():
    ws = xg.xgemm_workspace_bytes()
    for prec, shape, want in [("d", (8192, 8192, 8192), "d_128x128x16_w2x2"), ("d", (4096, 4096, 4096), "d_128x128x16_w2x2"),
                              ("s", (8192, 8192, 8192), "s_256x128x16_w2x2"), ("s", (16384, 16384, 16384), "s_256x128x16_w2x2"),
                              # rank-k updates: the smaller tile, three workgroups per CU to hide each other's flush of C
                              ("d", (16384, 16384, 64), "d_128x64x16_w2x2"), ("d", (16384, 16384, 256), "d_128x64x16_w2x2"),
                              ("d", (16384, 16384, 1024), "d_128x128x16_w2x2")]:
        for lwork in (0, ws):
            v, pieces, whole = xg.xgemm_plan(prec, 0, *shape, lwork)
            assert name(prec, v) == want and pieces == 1, (prec, shape, lwork)
            mt = [int(x) for x in want.split("_")[1].split("x")[:2]]
            assert whole == -(-shape[0] // mt[0]) * -(-shape[1] // mt[1])


def test_small_problems_take_small_tiles():
    # one matrix-instruction tile per wave: 32x32 tiles in fp64 (16x16x4), 64x64 in fp32 (32x32x2)
    for prec, tile, count in (("d", "32x32", 256), ("s", "64x64", 64)):
        v, pieces, whole = xg.xgemm_plan(prec, 0, 512, 512, 512, 0)
        assert name(prec, v).startswith(f"{prec}_{tile}") and pieces == 1 and whole == count
    v, pieces, whole = xg.xgemm_plan("d", 0, 1024, 1024, 1024, 0)
    assert name("d", v).startswith("d_64x64") and whole == 256


def test_tail_round_is_split_only_with_a_workspace_and_only_the_tail():
    ws = xg.xgemm_workspace_bytes()
    # 26 x 20 = 520 tiles of 128 x 128 on 512 slots
    v, pieces, whole = xg.xgemm_plan("d", 0, 3328, 2560, 2048, ws)
    assert name("d", v) == "d_128x128x16_w2x2" and pieces > 1 and whole == 512
    assert xg.xgemm_plan("d", 0, 3328, 2560, 2048, 0)[1] == 1
    assert xg.xgemm_plan("d", 0, 3328, 2560, 2048, 8192)[1] == 1            # counters only: no room for partial tiles
    # depth limits the pieces: at least 4 slabs of 16 each
    assert xg.xgemm_plan("d", 0, 3328, 2560, 128, ws)[1] <= 2
    # a tall-K product with few tiles is split from the first tile on
    v, pieces, whole = xg.xgemm_plan("d", 0, 512, 512, 8192, ws)
    assert name("d", v) == "d_128x128x16_w2x2" and pieces >= 8 and whole == 0
    # the triangular update counts the tiles of the triangle only
    v, pieces, whole = xg.xgemm_plan("d", 1, 8192, 8192, 8192, ws)
    assert name("d", v) == "d_128x128x16_w2x2" and whole == 2048 and pieces == 8      # 2080 tiles: 32 in the tail


def test_without_a_workspace_the_tail_round_of_a_deep_product_runs_as_quarter_tiles():
    # the rank-8192 update of a triangle of order 8192: 2080 tiles of 128 x 128 on 512 slots,
    # four full rounds and 32 tiles that a second launch computes as 128 tiles of 64 x 64
    v, pieces, whole = xg.xgemm_plan("d", 1, 8192, 8192, 8192, 0)
    assert name("d", v) == "d_128x128x16_w2x2" and pieces == 1 and whole == 2048
    # 40 x 40 tiles: three full rounds and 64 tiles
    v, pieces, whole = xg.xgemm_plan("d", 0, 5120, 5120, 5120, 0)
    assert name("d", v) == "d_128x128x16_w2x2" and pieces == 1 and whole == 1536
    # shallow products are left alone unless the tuning control asks for it
    v, pieces, whole = xg.xgemm_plan("d", 0, 5120, 5120, 256, 0)
    mt = [int(x) for x in name("d", v).split("_")[1].split("x")[:2]]
    assert pieces == 1 and whole == (5120 // mt[0]) * (5120 // mt[1])
    xg.xgemm_force_variant(0)
    xg.xgemm_force_split(1)
    assert xg.xgemm_plan("d", 0, 5120, 5120, 256, 0) == (0, 1, 1536)
    xg.xgemm_force_split(0)
    assert xg.xgemm_plan("d", 0, 5120, 5120, 5120, 0) == (0, 1, 1600)
    # nothing to quarter: fewer tiles than one round, or a variant with no half-size partner
    xg.xgemm_force_split(1)
    assert xg.xgemm_plan("d", 0, 1024, 1024, 4096, 0) == (0, 1, 64)
    v32 = [i for i in range(16) if (name("d", i) or "").startswith("d_32x32")][0]
    xg.xgemm_force_variant(v32)
    assert xg.xgemm_plan("d", 0, 5120, 5120, 5120, 0) == (v32, 1, 25600)
    # 64x64 tiles have 32x32 quarters: 6400 tiles on 1024 slots, six full rounds and 256 tiles
    v64 = [i for i in range(16) if (name("d", i) or "").startswith("d_64x64")][0]
    xg.xgemm_force_variant(v64)
    assert xg.xgemm_plan("d", 0, 5120, 5120, 5120, 0) == (v64, 1, 6144)


def test_forcing_and_errors():
    ws = xg.xgemm_workspace_bytes()
    xg.xgemm_force_variant(3)
    assert xg.xgemm_plan("d", 0, 8192, 8192, 8192, ws)[0] == 3
    xg.xgemm_force_variant(0)
    xg.xgemm_force_split(0)
    assert xg.xgemm_plan("d", 0, 3328, 2560, 2048, ws)[1] == 1
    xg.xgemm_force_split(4)
    assert xg.xgemm_plan("d", 0, 3328, 2560, 2048, ws)[1] == 4
    assert xg.xgemm_plan("x", 0, 8, 8, 8, 0) == -1
    assert xg.xgemm_plan("d", 3, 8, 8, 8, 0) == -2
    assert xg.xgemm_plan("d", 0, 0, 8, 8, 0) == -3
    assert xg.xgemm_plan("d", 0, 8, 8, 0, 0) == -5


def test_picks_that_measurement_corrected():
    """Three picks the planner got wrong until its model was corrected against the forced variants (each of these
    was 6-15 % behind the best variant): a round of lone workgroups is priced per variant, and a quartered tail
    costs one launch plus the longer of the first launch's drain and its own time."""
    # 1280^3: 100 tiles of 128 x 128 or 200 of 128 x 64 would leave CUs idle or alone; 400 tiles of 64 x 64 win
    v, pieces, whole = xg.xgemm_plan("d", 0, 1280, 1280, 1280, 0)
    assert name("d", v) == "d_64x64x16_w2x2" and pieces == 1 and whole == 400
    # 3072^3: one full round of 128 x 128 tiles and 64 tiles as quarter tiles, in both precisions
    for prec in "ds":
        v, pieces, whole = xg.xgemm_plan(prec, 0, 3072, 3072, 3072, 0)
        assert name(prec, v) == f"{prec}_128x128x16_w2x2" and pieces == 1 and whole == 512
