"""GPU parity of the triangular product against the CPU oracle: the product
bound |B_out - alpha op(T) B| <= 4 dim u |alpha||op(T)||B| on every element,
bit-exact on integer data, padding and T untouched."""
import itertools

import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import to_dev, torch_mod, unit_roundoff

pytestmark = pytest.mark.gpu

FLAGS = list(itertools.product("LR", "LU", "NT", "NU"))
DTYPES = [np.float64, np.float32]


def run_trmm(side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb, expect=0):
    torch = torch_mod()
    f = xg.xgemm_dtrmm if B.dtype == np.float64 else xg.xgemm_strmm
    dA, dB = to_dev(A), to_dev(B)
    rc = f(side, uplo, trans, diag, m, n, alpha, dA, lda, dB, ldb)
    torch.cuda.synchronize()
    assert rc == expect, f"return code {rc}"
    if A is not None:
        assert np.array_equal(dA.cpu().numpy(), A, equal_nan=True), "T was modified"
    return dB.cpu().numpy()


def make(rng, side, uplo, diag, m, n, pad, dtype):
    dim = m if side == "L" else n
    lda, ldb = max(dim, 1) + pad[0], max(m, 1) + pad[1]
    A = si.uniform(rng, dim, dim, lda, dtype)
    si._mask_triangle(A, dim, uplo, diag == "U", np.nan)
    return A, lda, si.uniform(rng, m, n, ldb, dtype), ldb


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_all_variants_from_one_block_to_several_levels(dtype, side, uplo, trans, diag):
    rng = si.rng_for(140, FLAGS.index((side, uplo, trans, diag)))
    for (m, n), pad in zip([(37, 50), (64, 64), (100, 129), (517, 300), (300, 517), (1, 1), (65, 3)],
                           itertools.cycle([(0, 0), (3, 5)])):
        A, lda, B, ldb = make(rng, side, uplo, diag, m, n, pad, dtype)
        out = run_trmm(side, uplo, trans, diag, m, n, 1.5, A, lda, B, ldb)
        assert np.array_equal(out[:, m:], B[:, m:], equal_nan=True), "padding rows of B were written"
        info, E, G = oracle.trmm_ext(side, uplo, trans, diag, m, n, 1.5, A, lda, B, ldb)
        dim = m if side == "L" else n
        nviol, ratio = oracle.bound_violations(out[:, :m], E, G, dim, unit_roundoff(dtype), 4.0)
        assert info == 0 and nviol == 0, f"{side}{uplo}{trans}{diag} {m}x{n}: {nviol} outside the bound, ratio {ratio}"


@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_integer_inputs_bit_exact(dtype, R, side, uplo, trans, diag):
    rng = si.rng_for(141, FLAGS.index((side, uplo, trans, diag)))
    m, n = (300, 130) if side == "L" else (130, 300)
    dim = m if side == "L" else n
    A = si.integers(rng, dim, dim, dim + 1, dtype, R)
    si._mask_triangle(A, dim, uplo, diag == "U", np.nan)
    B = si.integers(rng, m, n, m + 3, dtype, R)
    for alpha in (1.0, -2.0):
        out = run_trmm(side, uplo, trans, diag, m, n, alpha, A, dim + 1, B, m + 3)
        want = B.copy()
        assert oracle.trmm_work(side, uplo, trans, diag, m, n, alpha, A, dim + 1, want, m + 3) == 0
        assert np.array_equal(out, want, equal_nan=True)


@pytest.mark.parametrize("dtype", DTYPES)
def test_scalar_paths(dtype):
    rng = si.rng_for(142, 0)
    m, n = 150, 70
    A, lda, B, ldb = make(rng, "L", "L", "N", m, n, (1, 2), dtype)
    nanB = np.full_like(B, np.nan)
    out = run_trmm("L", "L", "N", "N", m, n, 0.0, None, lda, nanB, ldb)
    assert np.all(out[:, :m] == 0) and np.all(np.isnan(out[:, m:]))
    eye = si.identity(m, lda, dtype)
    out = run_trmm("L", "U", "T", "N", m, n, 2.0, eye, lda, B, ldb)
    assert np.array_equal(out[:, :m], 2.0 * B[:, :m])
    assert run_trmm("R", "L", "N", "N", m, 0, 1.0, None, 1, B, ldb) is not None


@pytest.mark.parametrize("dtype,side,uplo,trans,diag,m,n",
                         [(np.float64, "L", "L", "N", "N", 4096, 4096), (np.float64, "R", "U", "T", "U", 2048, 4096),
                          (np.float32, "L", "U", "N", "N", 4096, 2048)])
def test_larger_sizes_against_the_product_oracle_on_sampled_entries(dtype, side, uplo, trans, diag, m, n):
    """Sampled entries through the general-product oracle on a densified copy of the
    triangle (zeros and ones filled in), which the pins show to be the same sum."""
    rng = si.rng_for(143, m + n)
    A, lda, B, ldb = make(rng, side, uplo, diag, m, n, (8, 8), dtype)
    out = run_trmm(side, uplo, trans, diag, m, n, -1.0, A, lda, B, ldb)
    dim = m if side == "L" else n
    S = np.nan_to_num(A[:, :dim], nan=0.0)                     # (col, row) layout
    S = np.triu(S) if uplo == "L" else np.tril(S)              # lower triangle of the matrix = upper of the layout
    if diag == "U":
        np.fill_diagonal(S, 1.0)
    Td = np.ascontiguousarray(S.astype(dtype))
    C0 = np.zeros((n, m), dtype=dtype)
    I, J = si.sample_indices(rng, m, n, 3, 3, 4096)
    if side == "L":
        info, cref, g = oracle.gemm_samples(trans, "N", m, n, m, -1.0, Td, dim, B, ldb, 0.0, C0, m, I, J)
    else:
        info, cref, g = oracle.gemm_samples("N", trans, m, n, n, -1.0, B, ldb, Td, dim, 0.0, C0, m, I, J)
    nviol, ratio = oracle.bound_violations(out[J, I], cref, g, dim, unit_roundoff(dtype), 4.0)
    assert info == 0 and nviol == 0, (nviol, ratio)
    assert np.array_equal(out[:, m:], B[:, m:], equal_nan=True)


@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("side,uplo,trans", [("L", "L", "N"), ("L", "U", "N"), ("R", "L", "N"), ("L", "L", "T")])
def test_every_order_of_a_single_diagonal_block_bit_exact(dtype, R, side, uplo, trans):
    """Orders 1..256 are one launch of a diagonal-block kernel each (two kernels, many code paths
    that depend on the order: ragged last tiles, ragged last panels, panels never fetched).  Integer
    data, so that every entry is compared exactly; repeated, because an earlier form of the order-256
    kernel (runtime jumps around whole tiles, which left the compiler's wait states short on the jumping
    path) showed wrong last rows for some orders in some runs only."""
    rng = si.rng_for(142, "LR".index(side) * 4 + "LU".index(uplo) * 2 + "NT".index(trans))
    nrhs = 70
    for dim in list(range(1, 257, 5)) + [64, 128, 176, 190, 191, 192, 208, 255, 256]:
        m, n = (dim, nrhs) if side == "L" else (nrhs, dim)
        A = si.integers(rng, dim, dim, dim + 1, dtype, R)
        si._mask_triangle(A, dim, uplo, False, np.nan)
        B = si.integers(rng, m, n, m + 3, dtype, R)
        want = B.copy()
        assert oracle.trmm_work(side, uplo, trans, "N", m, n, 1.0, A, dim + 1, want, m + 3) == 0
        for rep in range(3):
            out = run_trmm(side, uplo, trans, "N", m, n, 1.0, A, dim + 1, B, m + 3)
            assert np.array_equal(out, want, equal_nan=True), f"order {dim}, run {rep}"
