"""GPU parity of the quartered tail: without a workspace, the tiles of the last,
partly filled round of workgroups run as four quarter tiles each in a second
launch with the variant of half the tile size.  Shapes with a few tiles more
than fit the compute units, ragged edges, both triangles; integer data exact,
real data within the usual bound, nothing outside the result written."""
import itertools

import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import (check_full, check_syrk_full, make_operands, make_syrk_operands, run_real, run_syrk)

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto():
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)
    yield
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)


def tail_plan(prec, uplo, m, n, k):
    """Fix the 128x128 variant and the quartered tail (whatever the planner would rather do for products
    this shallow) and return (variant name, whole tiles, all tiles) of the plan without a workspace."""
    want = f"{prec}_128x128x16"
    idx = [v for v in range(16) if (xg.xgemm_variant_name(prec, v) or "").startswith(want)]
    assert idx and xg.xgemm_force_variant(idx[0]) == 0
    assert xg.xgemm_force_split(1) == 0
    v, pieces, whole = xg.xgemm_plan(prec, uplo, m, n, k, 0)
    name = xg.xgemm_variant_name(prec, v)
    mt_m, mt_n = (int(x) for x in name.split("_")[1].split("x")[:2])
    tm, tn = -(-m // mt_m), -(-n // mt_n)
    tiles = tm * tn if uplo == 0 else sum(1 for i in range(tm) for j in range(tn)
                                          if (i * mt_m + mt_m - 1 >= j * mt_n if uplo == 1 else j * mt_n + mt_n - 1 >= i * mt_m))
    assert pieces == 1
    return name, whole, tiles


@pytest.mark.parametrize("dtype,prec,R", [(np.float64, "d", 1000), (np.float32, "s", 8)])
@pytest.mark.parametrize("ta,tb", [("N", "N"), ("T", "T"), ("N", "T")])
def test_product_with_a_few_tiles_too_many_integer_exact(dtype, prec, R, ta, tb):
    rng = si.rng_for(220, "NT".index(ta) * 2 + "NT".index(tb))
    for (m, n, k), pad in [((3328, 2560, 256), (0, 0, 0)), ((3329, 2561, 200), (1, 3, 5))]:
        name, whole, tiles = tail_plan(prec, 0, m, n, k)
        assert 0 < whole < tiles, f"{name}: this shape is meant to have a quartered tail ({whole} of {tiles})"
        A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad, dtype, "int", R)
        out = run_real(xg, ta, tb, m, n, k, -1.0, A, lda, B, ldb, 1.0, C, ldc)
        want = C.copy()
        assert oracle.gemm_work(ta, tb, m, n, k, -1.0, A, lda, B, ldb, 1.0, want, ldc) == 0
        assert np.array_equal(out, want, equal_nan=True), f"{ta}{tb} {m}x{n}x{k}"


@pytest.mark.parametrize("dtype,prec", [(np.float64, "d"), (np.float32, "s")])
def test_product_real_data_full_check(dtype, prec):
    rng = si.rng_for(221, 0)
    m, n, k = 3400, 2500, 300
    name, whole, tiles = tail_plan(prec, 0, m, n, k)
    assert 0 < whole < tiles
    A, lda, B, ldb, C, ldc = make_operands(rng, "T", "N", m, n, k, (2, 0, 4), dtype)
    check_full(xg, "T", "N", m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc)


@pytest.mark.parametrize("dtype,prec", [(np.float64, "d"), (np.float32, "s")])
@pytest.mark.parametrize("uplo,trans", list(itertools.product("LU", "NT")))
def test_triangular_update_with_a_quartered_tail(dtype, prec, uplo, trans):
    rng = si.rng_for(222, "LU".index(uplo) * 2 + "NT".index(trans))
    n, k = 4200, 200
    name, whole, tiles = tail_plan(prec, 1 if uplo == "L" else 2, n, n, k)
    assert 0 < whole < tiles, f"{name}: {whole} of {tiles}"
    A, lda, C, ldc = make_syrk_operands(rng, trans, n, k, (3, 1), dtype)
    check_syrk_full(xg, uplo, trans, n, k, -1.0, A, lda, 1.0, C, ldc)
    # integer data: the triangle exactly, the rest untouched
    A, lda, C, ldc = make_syrk_operands(rng, trans, n, k, (0, 2), dtype, "int", 8)
    out = run_syrk(xg, uplo, trans, n, k, 1.0, A, lda, -1.0, C, ldc)
    want = C.copy()
    assert oracle.syrk_work(uplo, trans, n, k, 1.0, A, lda, -1.0, want, ldc) == 0
    assert np.array_equal(out, want, equal_nan=True)


@pytest.mark.parametrize("dtype,prec,R", [(np.float64, "d", 1000), (np.float32, "s", 8)])
@pytest.mark.parametrize("ta,tb", [("N", "N"), ("T", "T"), ("N", "T"), ("T", "N")])
def test_edge_tiles_whose_last_vector_straddles_the_edge(dtype, prec, R, ta, tb):
    """Edge tiles load full-depth slabs 16 bytes at a time; where the row or column count is no
    multiple of the vector, the last vector reaches past the edge into the padding (NaN here)
    or the next stored column.  Depths that are whole slabs (the last slab must not reach past
    the array) and ragged ones, tight and padded leading dimensions, operands narrower than a vector."""
    rng = si.rng_for(223, "NT".index(ta) * 2 + "NT".index(tb))
    shapes = [(129, 131, 64), (257, 67, 128), (131, 129, 50), (1, 1, 32), (2, 3, 32), (3, 2, 48), (5, 7, 16), (383, 255, 96)]
    for v in range(16):
        if xg.xgemm_variant_name(prec, v) is None:
            break
        assert xg.xgemm_force_variant(v) == 0
        for (m, n, k), pad in itertools.product(shapes, [(0, 0, 0), (1, 3, 2)]):
            A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad, dtype, "int", R)
            out = run_real(xg, ta, tb, m, n, k, 2.0, A, lda, B, ldb, -1.0, C, ldc)
            want = C.copy()
            assert oracle.gemm_work(ta, tb, m, n, k, 2.0, A, lda, B, ldb, -1.0, want, ldc) == 0
            assert np.array_equal(out, want, equal_nan=True), f"{xg.xgemm_variant_name(prec, v)} {ta}{tb} {m}x{n}x{k} pad {pad}"
