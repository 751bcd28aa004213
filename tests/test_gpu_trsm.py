"""GPU parity of the triangular solve against the CPU oracle.

A solve has no element-wise comparison that holds for every T (the forward error
grows with the condition number), so the unique, checkable statement is the
componentwise residual computed by the oracle in extended precision:
    |alpha B - op(T) X| <= 4 dim u (|alpha B| + |op(T)||X|),
which any summation order of the substitution satisfies.  Integer systems built
from a known integer solution must be recovered bit for bit, and X is also
compared with the oracle's own X on well-conditioned inputs."""
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


def run_trsm(side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb, expect=0):
    torch = torch_mod()
    f = xg.xgemm_dtrsm if B.dtype == np.float64 else xg.xgemm_strsm
    dA, dB = to_dev(A), to_dev(B)
    rc = f(side, uplo, trans, diag, m, n, alpha, dA, lda, dB, ldb)
    torch.cuda.synchronize()
    assert rc == expect, f"return code {rc}"
    if A is not None:
        assert np.array_equal(dA.cpu().numpy(), A, equal_nan=True), "T was modified"
    return dB.cpu().numpy()


def make(rng, side, uplo, diag, m, n, pad=(0, 0), dtype=np.float64):
    dim = m if side == "L" else n
    lda, ldb = max(dim, 1) + pad[0], max(m, 1) + pad[1]
    return si.triangular(rng, dim, lda, dtype, uplo, diag == "U"), lda, si.uniform(rng, m, n, ldb, dtype), ldb


def check(side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb):
    X = run_trsm(side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb)
    assert np.array_equal(X[:, m:], B[:, m:], equal_nan=True), "padding rows of B were written"
    info, R, G = oracle.trsm_resid(side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb, X, ldb)
    assert info == 0
    dim = m if side == "L" else n
    bound = 4.0 * dim * unit_roundoff(B.dtype) * G
    assert np.all(np.isfinite(X[:, :m])) and np.all(np.abs(R) <= bound), \
        f"{side}{uplo}{trans}{diag} {m}x{n}: max ratio {float(np.max(np.abs(R) / np.maximum(bound, 1e-300)))}"
    # the generator's matrices are well conditioned: X itself agrees with the oracle's substitution
    want = B.copy()
    assert oracle.trsm_work(side, uplo, trans, diag, m, n, alpha, A, lda, want, ldb) == 0
    tol = 64 * dim * unit_roundoff(B.dtype)
    assert np.allclose(X[:, :m], want[:, :m], rtol=tol, atol=tol)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_all_variants_from_one_block_to_several_levels(dtype, side, uplo, trans, diag):
    rng = si.rng_for(120, FLAGS.index((side, uplo, trans, diag)))
    # one diagonal block; exactly one block; two blocks with a ragged second; several levels, ragged
    for (m, n), pad in zip([(37, 50), (64, 64), (100, 129), (517, 300), (300, 517), (1, 1), (65, 3)],
                           itertools.cycle([(0, 0), (3, 5)])):
        A, lda, B, ldb = make(rng, side, uplo, diag, m, n, pad, dtype)
        check(side, uplo, trans, diag, m, n, 1.5, A, lda, B, ldb)


@pytest.mark.parametrize("dtype,R", [(np.float64, 4), (np.float32, 2)])
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_integer_systems_bit_exact(dtype, R, side, uplo, trans, diag):
    rng = si.rng_for(121, FLAGS.index((side, uplo, trans, diag)))
    m, n = (300, 130) if side == "L" else (130, 300)
    dim = m if side == "L" else n
    A = si.int_triangular(rng, dim, dim + 1, dtype, uplo, diag == "U", R)
    Xtrue = rng.integers(-R, R + 1, size=(m, n)).astype(np.int64)
    S = np.nan_to_num(si.view(A, dim), nan=0.0).astype(np.int64)
    T = np.tril(S) if uplo == "L" else np.triu(S)
    if diag == "U":
        np.fill_diagonal(T, 1)
    T = T.T if trans == "T" else T
    Bint = T @ Xtrue if side == "L" else Xtrue @ T
    B = si.constant(m, n, m + 3, dtype)
    B[:, :m] = Bint.T.astype(dtype)
    X = run_trsm(side, uplo, trans, diag, m, n, 1.0, A, dim + 1, B, m + 3)
    assert np.array_equal(X[:, :m], Xtrue.T.astype(dtype))
    want = B.copy()
    assert oracle.trsm_work(side, uplo, trans, diag, m, n, 1.0, A, dim + 1, want, m + 3) == 0
    assert np.array_equal(X, want, equal_nan=True)


@pytest.mark.parametrize("dtype", DTYPES)
def test_scalar_paths(dtype):
    rng = si.rng_for(122, 0)
    m, n = 150, 70
    A, lda, B, ldb = make(rng, "L", "L", "N", m, n, (1, 2), dtype)
    # alpha == 0: X = 0 whatever B held, T not read
    nanB = np.full_like(B, np.nan)
    X = run_trsm("L", "L", "N", "N", m, n, 0.0, None, lda, nanB, ldb)
    assert np.all(X[:, :m] == 0) and np.all(np.isnan(X[:, m:]))
    # identity with alpha: X = alpha B exactly
    eye = si.identity(m, lda, dtype)
    X = run_trsm("L", "U", "T", "N", m, n, 2.0, eye, lda, B, ldb)
    assert np.array_equal(X[:, :m], 2.0 * B[:, :m])
    # empty problems return at once
    assert run_trsm("R", "L", "N", "N", m, 0, 1.0, None, 1, B, ldb) is not None


@pytest.mark.parametrize("dtype,side,uplo,trans,diag,m,n",
                         [(np.float64, "L", "L", "N", "N", 8192, 8192), (np.float64, "R", "U", "N", "N", 4096, 8192),
                          (np.float64, "L", "U", "T", "U", 4096, 4096), (np.float32, "R", "L", "T", "N", 8192, 4096),
                          (np.float32, "L", "L", "N", "U", 8192, 8192)])
def test_full_size_sampled_residual(dtype, side, uplo, trans, diag, m, n):
    rng = si.rng_for(123, m + n)
    A, lda, B, ldb = make(rng, side, uplo, diag, m, n, (8, 8), dtype)
    X = run_trsm(side, uplo, trans, diag, m, n, -1.0, A, lda, B, ldb)
    assert np.all(np.isfinite(X[:, :m]))
    I, J = si.sample_indices(rng, m, n, 4, 4, 8192)
    info, R, G = oracle.trsm_resid_samples(side, uplo, trans, diag, m, n, -1.0, A, lda, B, ldb, X, ldb, I, J)
    assert info == 0
    dim = m if side == "L" else n
    assert np.all(np.abs(R) <= 4.0 * dim * unit_roundoff(dtype) * G)
    assert np.array_equal(X[:, m:], B[:, m:], equal_nan=True)


@pytest.mark.parametrize("dtype,side,dim,nrhs",
                         [(np.float64, "L", 50, 9000), (np.float64, "R", 64, 17000), (np.float64, "L", 200, 5000),
                          (np.float64, "R", 256, 9000), (np.float64, "L", 250, 3000), (np.float64, "R", 256, 700),
                          (np.float32, "L", 60, 17000), (np.float32, "R", 33, 33000), (np.float32, "L", 130, 17000),
                          (np.float32, "R", 256, 3000), (np.float32, "L", 200, 5000), (np.float32, "R", 256, 10000),
                          (np.float64, "L", 200, 17000), (np.float32, "R", 256, 17000)])
def test_many_right_hand_sides_on_one_small_triangle(dtype, side, dim, nrhs):
    """The diagonal-block kernels pack 2 to 16 right-hand sides into a wave, and the one for orders
    up to 256 runs with or without separate feeding waves, depending on how many right-hand sides
    there are; these counts reach the combinations that the other cases do not."""
    rng = si.rng_for(124, dim + nrhs)
    m, n = (dim, nrhs) if side == "L" else (nrhs, dim)
    for uplo, trans in (("L", "N"), ("U", "T")):
        A, lda, B, ldb = make(rng, side, uplo, "N", m, n, (3, 5), dtype)
        X = run_trsm(side, uplo, trans, "N", m, n, 0.75, A, lda, B, ldb)
        assert np.all(np.isfinite(X[:, :m]))
        I, J = si.sample_indices(rng, m, n, 4, 4, 8192)
        info, R, G = oracle.trsm_resid_samples(side, uplo, trans, "N", m, n, 0.75, A, lda, B, ldb, X, ldb, I, J)
        assert info == 0
        assert np.all(np.abs(R) <= 4.0 * dim * unit_roundoff(dtype) * G)
        assert np.array_equal(X[:, m:], B[:, m:], equal_nan=True)


@pytest.mark.parametrize("dtype,R", [(np.float64, 4), (np.float32, 2)])
@pytest.mark.parametrize("side,uplo,trans", [("L", "L", "N"), ("L", "U", "N"), ("R", "L", "N"), ("L", "L", "T")])
def test_every_order_of_a_single_diagonal_block_bit_exact(dtype, R, side, uplo, trans):
    """Orders 1..256 are one launch of a diagonal-block kernel each (order <= 64: the block in LDS;
    above: panels through LDS, with code paths that depend on the order).  Integer systems with a
    known integer solution, recovered exactly, each order three times."""
    rng = si.rng_for(125, "LR".index(side) * 4 + "LU".index(uplo) * 2 + "NT".index(trans))
    nrhs = 70
    for dim in list(range(1, 257, 5)) + [64, 128, 176, 190, 191, 192, 208, 255, 256]:
        m, n = (dim, nrhs) if side == "L" else (nrhs, dim)
        A = si.int_triangular(rng, dim, dim + 1, dtype, uplo, False, R)
        Xtrue = rng.integers(-R, R + 1, size=(m, n)).astype(np.int64)
        S = np.nan_to_num(si.view(A, dim), nan=0.0).astype(np.int64)
        T = np.tril(S) if uplo == "L" else np.triu(S)
        T = T.T if trans == "T" else T
        Bint = T @ Xtrue if side == "L" else Xtrue @ T
        if np.abs(Bint).max() >= (2 ** 52 if dtype == np.float64 else 2 ** 23):
            continue                                   # right-hand side not exactly representable
        B = si.constant(m, n, m + 3, dtype)
        B[:, :m] = Bint.T.astype(dtype)
        for rep in range(3):
            X = run_trsm(side, uplo, trans, "N", m, n, 1.0, A, dim + 1, B, m + 3)
            assert np.array_equal(X[:, :m], Xtrue.T.astype(dtype)), f"order {dim}, run {rep}"
