"""Pins for the triangular-solve oracle: exact rationals on tiny systems, integer
systems with known integer solutions, a library routine as a third opinion,
closed forms, the parts of T that must not be read, scalar paths, error codes,
and the residual routine itself."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.linalg

import oracle
import synth_inputs as si

FLAGS = list(itertools.product("LR", "LU", "NT", "NU"))


def dense_op_T(A, dim, uplo, trans, diag):
    """op(T) as a dense (row, col) array built from the stored triangle only."""
    S = si.view(A, dim).copy()
    T = np.tril(S) if uplo == "L" else np.triu(S)
    T = np.nan_to_num(T, nan=0.0)
    if diag == "U":
        np.fill_diagonal(T, 1.0)
    return T.T if trans == "T" else T


def make(rng, side, uplo, diag, m, n, pad=(0, 0), dtype=np.float64):
    dim = m if side == "L" else n
    lda, ldb = max(dim, 1) + pad[0], max(m, 1) + pad[1]
    A = si.triangular(rng, dim, lda, dtype, uplo, diag == "U")
    B = si.uniform(rng, m, n, ldb, dtype)
    return A, lda, B, ldb


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_tiny_systems_against_exact_rationals(side, uplo, trans, diag):
    rng = si.rng_for(110, 1)
    for m, n in [(1, 1), (2, 3), (3, 2), (5, 4), (4, 5)]:
        A, lda, B, ldb = make(rng, side, uplo, diag, m, n, (1, 2))
        alpha = 1.5
        X = B.copy()
        assert oracle.trsm_work(side, uplo, trans, diag, m, n, alpha, A, lda, X, ldb) == 0
        assert np.all(np.isnan(X[:, m:]))                      # padding untouched
        dim = m if side == "L" else n
        T = dense_op_T(A, dim, uplo, trans, diag)
        Fr = lambda M: [[Fraction(float(v)) for v in row] for row in M]
        Tq, Xq, Bq = Fr(T), Fr(si.view(X, m)), Fr(si.view(B, m))
        for i in range(m):
            for j in range(n):
                if side == "L":
                    terms = [Tq[i][c] * Xq[c][j] for c in range(m)]
                else:
                    terms = [Xq[i][c] * Tq[c][j] for c in range(n)]
                rhs = Fraction(alpha) * Bq[i][j]
                resid = abs(rhs - sum(terms, Fraction(0)))
                scale = abs(rhs) + sum((abs(t) for t in terms), Fraction(0))
                # componentwise backward error of substitution: gamma_(dim+1), taken with slack
                assert resid <= Fraction(oracle.U64) * (dim + 2) * scale


@pytest.mark.parametrize("dtype,R", [(np.float64, 4), (np.float32, 2)])
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_integer_systems_recover_the_integer_solution_exactly(dtype, R, side, uplo, trans, diag):
    rng = si.rng_for(110, 2)
    m, n = 37, 29
    dim = m if side == "L" else n
    A = si.int_triangular(rng, dim, dim + 3, dtype, uplo, diag == "U", R)
    Xtrue = rng.integers(-R, R + 1, size=(m, n)).astype(np.int64)
    T = dense_op_T(A, dim, uplo, trans, diag).astype(np.int64)
    Bint = T @ Xtrue if side == "L" else Xtrue @ T
    B = si.constant(m, n, m + 2, dtype)
    B[:, :m] = Bint.T.astype(dtype)
    assert oracle.trsm_work(side, uplo, trans, diag, m, n, 1.0, A, dim + 3, B, m + 2) == 0
    assert np.array_equal(si.view(B, m), Xtrue.astype(dtype))


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_against_library_triangular_solver(side, uplo, trans, diag):
    rng = si.rng_for(110, 3)
    m, n = 61, 45
    A, lda, B, ldb = make(rng, side, uplo, diag, m, n, (2, 1))
    X = B.copy()
    assert oracle.trsm_work(side, uplo, trans, diag, m, n, -0.75, A, lda, X, ldb) == 0
    dim = m if side == "L" else n
    T = dense_op_T(A, dim, uplo, trans, diag)
    rhs = -0.75 * si.view(B, m)
    lower = (uplo == "L") != (trans == "T")
    if side == "L":
        want = scipy.linalg.solve_triangular(T, rhs, lower=lower)
    else:
        want = scipy.linalg.solve_triangular(T.T, rhs.T, lower=not lower).T
    assert np.allclose(si.view(X, m), want, rtol=1e-12, atol=1e-13)


def test_closed_forms_and_scalar_paths():
    rng = si.rng_for(110, 4)
    m, n = 9, 7
    B = si.uniform(rng, m, n, m + 1)
    for side, dim in (("L", m), ("R", n)):
        # identity: X = alpha B; unit diagonal with a NaN stored diagonal and NaN other triangle
        A = np.full((dim, dim), np.nan)
        A[np.tril_indices(dim, -1)[::-1]] = 0.0      # strictly lower part in (col, row) layout
        X = B.copy()
        assert oracle.trsm_work(side, "L", "N", "U", m, n, 2.0, A, dim, X, m + 1) == 0
        assert np.array_equal(X[:, :m], 2.0 * B[:, :m])
        # diagonal matrix: element-wise quotient
        d = rng.uniform(1, 2, size=dim)
        A = np.diag(d)
        X = B.copy()
        assert oracle.trsm_work(side, "U", "T", "N", m, n, 1.0, A, dim, X, m + 1) == 0
        want = B[:, :m] / (d[None, :] if side == "L" else d[:, None])
        assert np.array_equal(X[:, :m], want)
    # alpha == 0: X = 0, neither T nor B's values matter
    X = np.full((n, m + 1), np.nan)
    assert oracle.trsm_work("L", "L", "N", "N", m, n, 0.0, None, m, X, m + 1) == 0
    assert np.all(X[:, :m] == 0) and np.all(np.isnan(X[:, m:]))
    # empty problems
    assert oracle.trsm_work("L", "L", "N", "N", 0, n, 1.0, None, 1, None, 1) == 0
    assert oracle.trsm_work("R", "L", "N", "N", m, 0, 1.0, None, 1, None, m) == 0


def test_errors():
    A = np.eye(4)
    B = np.ones((3, 4))
    t = oracle.trsm_work
    assert t("X", "L", "N", "N", 4, 3, 1.0, A, 4, B, 4) == -1
    assert t("L", "X", "N", "N", 4, 3, 1.0, A, 4, B, 4) == -2
    assert t("L", "L", "X", "N", 4, 3, 1.0, A, 4, B, 4) == -3
    assert t("L", "L", "N", "X", 4, 3, 1.0, A, 4, B, 4) == -4
    assert t("L", "L", "N", "N", -1, 3, 1.0, A, 4, B, 4) == -5
    assert t("L", "L", "N", "N", 4, -1, 1.0, A, 4, B, 4) == -6
    assert t("L", "L", "N", "N", 4, 3, 1.0, None, 4, B, 4) == -8
    assert t("L", "L", "N", "N", 4, 3, 1.0, A, 3, B, 4) == -9
    assert t("R", "L", "N", "N", 4, 3, 1.0, A, 2, B, 4) == -9
    assert t("L", "L", "N", "N", 4, 3, 1.0, A, 4, None, 4) == -10
    assert t("L", "L", "N", "N", 4, 3, 1.0, A, 4, B, 3) == -11


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_residual_routine(side, uplo, trans, diag):
    """The residual of the oracle's own solution is within the substitution bound, it
    equals a dense evaluation, and a perturbed solution is caught."""
    rng = si.rng_for(110, 5)
    m, n = 33, 21
    A, lda, B, ldb = make(rng, side, uplo, diag, m, n, (1, 1))
    X = B.copy()
    assert oracle.trsm_work(side, uplo, trans, diag, m, n, 1.5, A, lda, X, ldb) == 0
    info, R, G = oracle.trsm_resid(side, uplo, trans, diag, m, n, 1.5, A, lda, B, ldb, X, ldb)
    assert info == 0
    dim = m if side == "L" else n
    assert np.all(np.abs(R) <= (dim + 2) * oracle.U64 * G)
    T = dense_op_T(A, dim, uplo, trans, diag).astype(np.longdouble)
    Xd, Bd = si.view(X, m).astype(np.longdouble), si.view(B, m).astype(np.longdouble)
    dense = np.longdouble(1.5) * Bd - (T @ Xd if side == "L" else Xd @ T)
    denseG = np.abs(np.longdouble(1.5) * Bd) + (np.abs(T) @ np.abs(Xd) if side == "L" else np.abs(Xd) @ np.abs(T))
    assert np.allclose(R.T, dense, rtol=0, atol=1e-17) and np.allclose(G.T, denseG, rtol=1e-15)
    I, J = si.sample_indices(rng, m, n, 3, 3, 200)
    info, Rs, Gs = oracle.trsm_resid_samples(side, uplo, trans, diag, m, n, 1.5, A, lda, B, ldb, X, ldb, I, J)
    assert info == 0 and np.array_equal(Rs, R[J, I]) and np.array_equal(Gs, G[J, I])
    assert oracle.trsm_resid_samples(side, uplo, trans, diag, m, n, 1.5, A, lda, B, ldb, X, ldb, [m], [0])[0] == -15
    Xbad = X.copy()
    Xbad[n // 2, m // 2] *= 1 + 1e-9
    _, R2, G2 = oracle.trsm_resid(side, uplo, trans, diag, m, n, 1.5, A, lda, B, ldb, Xbad, ldb)
    assert np.any(np.abs(R2) > 4 * dim * oracle.U64 * G2)
