"""GPU parity of the symmetric product and the rank-2k update against the CPU
oracle: the product bound with the number of terms of each element (dim for
symm, 2k for syr2k), bit-exact on integer data, nothing outside the result
written, the unreferenced triangle of the symmetric matrix never read (NaN)."""
import itertools

import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import to_dev, torch_mod, unit_roundoff

pytestmark = pytest.mark.gpu

DTYPES = [np.float64, np.float32]


def sym_matrix(rng, dim, ld, uplo, dtype, kind="uniform", R=8):
    A = si.uniform(rng, dim, dim, ld, dtype) if kind == "uniform" else si.integers(rng, dim, dim, ld, dtype, R)
    return si._mask_triangle(A, dim, uplo, False, np.nan)


def run(name, dtype, *args):
    torch = torch_mod()
    f = getattr(xg, f"xgemm_{'d' if dtype == np.float64 else 's'}{name}")
    f1, f2, d1, d2, alpha, A, lda, B, ldb, beta, C, ldc = args
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    assert f(f1, f2, d1, d2, alpha, dA, lda, dB, ldb, beta, dC, ldc) == 0
    torch.cuda.synchronize()
    return dC.cpu().numpy()


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("side,uplo", list(itertools.product("LR", "LU")))
def test_symm_from_one_block_to_several_levels(dtype, side, uplo):
    rng = si.rng_for(210, "LR".index(side) * 2 + "LU".index(uplo))
    for (m, n), pad, (alpha, beta) in zip([(37, 50), (64, 64), (100, 129), (517, 300), (300, 517), (1, 1), (65, 3)],
                                          itertools.cycle([(0, 0, 0), (3, 5, 2)]),
                                          itertools.cycle([(1.5, -0.5), (1.0, 0.0), (-1.0, 1.0)])):
        dim = m if side == "L" else n
        lda, ldb, ldc = dim + pad[0], m + pad[1], m + pad[2]
        A = sym_matrix(rng, dim, lda, uplo, dtype)
        B, C = si.uniform(rng, m, n, ldb, dtype), si.uniform(rng, m, n, ldc, dtype)
        if beta == 0.0:
            C[:, :m] = np.nan
        out = run("symm", dtype, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc)
        info, E, G = oracle.symm_ext(side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc)
        nviol, ratio = oracle.bound_violations(out[:, :m], E, G, dim, unit_roundoff(dtype), 4.0)
        assert info == 0 and nviol == 0, f"{side}{uplo} {m}x{n}: {nviol} outside the bound, ratio {ratio}"
        assert np.array_equal(out[:, m:], C[:, m:], equal_nan=True), "padding rows of C were written"


@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("side,uplo", list(itertools.product("LR", "LU")))
@pytest.mark.parametrize("dim,other", [(300, 130), (1030, 200), (768, 257), (513, 1)])
def test_symm_integer_bit_exact(dtype, R, side, uplo, dim, other):
    """Order 300: the recursion down to the block kernels.  Orders from 512 on: two products whose
    depth per tile stops short of (starts beyond) the tile's diagonal block, then the diagonal blocks;
    a ragged last diagonal block (1030) and a whole number of them (768).  The unreferenced triangle
    holds NaN throughout."""
    rng = si.rng_for(211, dim)
    m, n = (dim, other) if side == "L" else (other, dim)
    A = sym_matrix(rng, dim, dim + 1, uplo, dtype, "int", R)
    B, C = si.integers(rng, m, n, m + 2, dtype, R), si.integers(rng, m, n, m + 3, dtype, R)
    for alpha, beta in [(1.0, 0.0), (-2.0, 1.0), (1.0, -1.0)]:
        out = run("symm", dtype, side, uplo, m, n, alpha, A, dim + 1, B, m + 2, beta, C, m + 3)
        want = C.copy()
        assert oracle.symm_work(side, uplo, m, n, alpha, A, dim + 1, B, m + 2, beta, want, m + 3) == 0
        assert np.array_equal(out, want, equal_nan=True)


@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("side,uplo", [("L", "L"), ("R", "U")])
def test_symm_every_order_of_a_single_diagonal_block_bit_exact(dtype, R, side, uplo):
    """Orders 1..256 are one launch of a diagonal-block kernel each; integer data, every entry
    compared exactly, each order run three times (see the same test of the triangular product)."""
    rng = si.rng_for(212, "LR".index(side))
    other = 70
    for dim in list(range(1, 257, 5)) + [64, 128, 176, 190, 191, 192, 208, 255, 256]:
        m, n = (dim, other) if side == "L" else (other, dim)
        A = sym_matrix(rng, dim, dim + 1, uplo, dtype, "int", R)
        B, C = si.integers(rng, m, n, m + 2, dtype, R), si.integers(rng, m, n, m + 3, dtype, R)
        want = C.copy()
        assert oracle.symm_work(side, uplo, m, n, 1.0, A, dim + 1, B, m + 2, 1.0, want, m + 3) == 0
        for rep in range(3):
            out = run("symm", dtype, side, uplo, m, n, 1.0, A, dim + 1, B, m + 2, 1.0, C, m + 3)
            assert np.array_equal(out, want, equal_nan=True), f"order {dim}, run {rep}"


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("uplo,trans", list(itertools.product("LU", "NT")))
def test_syr2k_ragged_and_integer(dtype, uplo, trans):
    rng = si.rng_for(212, "LU".index(uplo) * 2 + "NT".index(trans))
    for (n, k), pad in zip([(300, 83), (1, 1), (129, 16), (515, 37)], itertools.cycle([(0, 0, 0), (3, 1, 5)])):
        ra, ca = (n, k) if trans == "N" else (k, n)
        lda, ldb, ldc = ra + pad[0], ra + pad[1], n + pad[2]
        A, B, C = si.uniform(rng, ra, ca, lda, dtype), si.uniform(rng, ra, ca, ldb, dtype), si.uniform(rng, n, n, ldc, dtype)
        out = run("syr2k", dtype, uplo, trans, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc)
        info, E, G = oracle.syr2k_ext(uplo, trans, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc)
        mask = oracle.triangle_mask(uplo, n)
        got = np.where(mask, out[:, :n], 0).astype(dtype)
        nviol, ratio = oracle.bound_violations(got, E, G, 2 * k, unit_roundoff(dtype), 4.0)
        assert info == 0 and nviol == 0, (n, k, nviol, ratio)
        keep = np.ones(C.shape, dtype=bool)
        keep[:, :n] = ~mask
        assert np.array_equal(out[keep], C[keep], equal_nan=True), "elements outside the triangle were written"
    R = 1000 if dtype == np.float64 else 8
    n, k = 384, 96
    ra, ca = (n, k) if trans == "N" else (k, n)
    A, B = si.integers(rng, ra, ca, ra, dtype, R), si.integers(rng, ra, ca, ra + 1, dtype, R)
    C = si.integers(rng, n, n, n + 1, dtype, R)
    out = run("syr2k", dtype, uplo, trans, n, k, 2.0, A, ra, B, ra + 1, -1.0, C, n + 1)
    want = C.copy()
    assert oracle.syr2k_work(uplo, trans, n, k, 2.0, A, ra, B, ra + 1, -1.0, want, n + 1) == 0
    assert np.array_equal(out, want, equal_nan=True)


def test_scalar_paths():
    torch = torch_mod()
    rng = si.rng_for(213, 0)
    m, n = 150, 70
    B, C = si.uniform(rng, m, n, m + 1), si.uniform(rng, m, n, m + 2)
    dC = to_dev(C)
    # alpha == 0: A and B unread, C := beta C
    assert xg.xgemm_dsymm("L", "U", m, n, 0.0, None, m, None, m + 1, 2.0, dC, m + 2) == 0
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    assert np.array_equal(out[:, :m], 2.0 * C[:, :m]) and np.array_equal(out[:, m:], C[:, m:], equal_nan=True)
    # identity: C := alpha B exactly with beta == 0 over NaN
    eye = to_dev(si.identity(m, m))
    dC = to_dev(np.full_like(C, np.nan))
    assert xg.xgemm_dsymm("L", "L", m, n, 2.0, eye, m, to_dev(B), m + 1, 0.0, dC, m + 2) == 0
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy()[:, :m], 2.0 * B[:, :m])


@pytest.mark.parametrize("name", ["symm", "syr2k"])
def test_4096_sampled(name):
    """Sampled entries through the general-product oracle (the pins show the sums to be the same)."""
    rng = si.rng_for(214, 0)
    n = 4096
    I, J = si.sample_indices(rng, n, n, 3, 3, 4096)
    if name == "symm":
        A = sym_matrix(rng, n, n, "L", np.float64)
        B, C = si.uniform(rng, n, n), si.uniform(rng, n, n)
        out = run("symm", np.float64, "L", "L", n, n, 1.5, A, n, B, n, -0.5, C, n)
        S = np.nan_to_num(A, nan=0.0)                # (col, row): lower triangle of the matrix = upper of the layout
        full = np.ascontiguousarray(S + S.T - np.diag(np.diag(S)))
        info, cref, g = oracle.gemm_samples("N", "N", n, n, n, 1.5, full, n, B, n, -0.5, C, n, I, J)
        nviol, ratio = oracle.bound_violations(out[J, I], cref, g, n, oracle.U64, 4.0)
    else:
        k = 2048
        A, B, C = si.uniform(rng, n, k), si.uniform(rng, n, k), si.uniform(rng, n, n)
        out = run("syr2k", np.float64, "U", "N", n, k, 1.5, A, n, B, n, -0.5, C, n)
        up = I <= J
        I, J = np.where(up, I, J), np.where(up, J, I)
        Z = np.zeros((n, n))
        info, c1, g1 = oracle.gemm_samples("N", "T", n, n, k, 1.5, A, n, B, n, -0.5, C, n, I, J)
        info2, c2, g2 = oracle.gemm_samples("N", "T", n, n, k, 1.5, B, n, A, n, 0.0, Z, n, I, J)
        assert info2 == 0
        nviol, ratio = oracle.bound_violations(out[J, I], c1 + c2, g1 + g2, 2 * k, oracle.U64, 4.0)
    assert info == 0 and nviol == 0, ratio


@pytest.mark.parametrize("dtype,prec,R", [(np.float64, "d", 1000), (np.float32, "s", 8)])
@pytest.mark.parametrize("side,uplo", [("L", "L"), ("R", "U")])
def test_symm_flat_passes_with_every_tile_variant(dtype, prec, R, side, uplo):
    """The two products with a depth range per tile, forced through every tile variant in turn (the range is
    taken from the tile's first row or column, so every tile size has to land on the block boundaries)."""
    rng = si.rng_for(213, 0)
    dim, other = 1030, 150
    m, n = (dim, other) if side == "L" else (other, dim)
    A = sym_matrix(rng, dim, dim + 1, uplo, dtype, "int", R)
    B, C = si.integers(rng, m, n, m + 2, dtype, R), si.integers(rng, m, n, m + 3, dtype, R)
    want = C.copy()
    assert oracle.symm_work(side, uplo, m, n, -1.0, A, dim + 1, B, m + 2, 1.0, want, m + 3) == 0
    try:
        for v in range(16):
            if xg.xgemm_variant_name(prec, v) is None:
                break
            assert xg.xgemm_force_variant(v) == 0
            out = run("symm", dtype, side, uplo, m, n, -1.0, A, dim + 1, B, m + 2, 1.0, C, m + 3)
            assert np.array_equal(out, want, equal_nan=True), xg.xgemm_variant_name(prec, v)
    finally:
        xg.xgemm_force_variant(-1)
