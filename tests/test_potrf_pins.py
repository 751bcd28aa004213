"""Pins for the Cholesky oracle: integer factors recovered exactly, a library
routine as a third opinion, closed forms, the residual bound, failure reporting,
the triangle that must stay untouched, error codes."""
import numpy as np
import pytest

import oracle
import synth_inputs as si


def int_factor(rng, n, R=3):
    """Integer lower-triangular L0 with a diagonal of powers of two (square roots and quotients exact)."""
    L0 = np.tril(rng.integers(-R, R + 1, size=(n, n)), -1).astype(np.int64)
    L0[np.arange(n), np.arange(n)] = 2 ** rng.integers(0, 3, size=n)
    return L0


def store(M, uplo, ld, dtype=np.float64):
    """Column-major storage of the `uplo` triangle of the (row, col) matrix M; NaN elsewhere."""
    n = M.shape[0]
    X = np.full((n, ld), np.nan, dtype=dtype)
    X[:, :n] = M.T.astype(dtype)
    return si._mask_triangle(X, n, uplo, False, np.nan)


@pytest.mark.parametrize("dtype,R", [(np.float64, 3), (np.float32, 2)])
@pytest.mark.parametrize("uplo", "LU")
def test_integer_factor_recovered_exactly(dtype, R, uplo):
    rng = si.rng_for(160, 1)
    n = 45
    L0 = int_factor(rng, n, R)
    A = store(L0 @ L0.T, uplo, n + 3, dtype)
    keep = A.copy()
    assert oracle.potrf(uplo, n, A, n + 3) == 0
    want = store(L0 if uplo == "L" else L0.T, uplo, n + 3, dtype)
    assert np.array_equal(A, want, equal_nan=True)          # factor exact; other triangle and padding still NaN
    assert np.array_equal(np.isnan(A), np.isnan(keep))


@pytest.mark.parametrize("uplo", "LU")
def test_against_library_cholesky_and_residual_bound(uplo):
    rng = si.rng_for(160, 2)
    n = 83
    A = si.spd(rng, n, n + 2, np.float64, uplo)
    F = A.copy()
    assert oracle.potrf(uplo, n, F, n + 2) == 0
    S = np.nan_to_num(si.view(A, n), nan=0.0)
    full = S + S.T - np.diag(np.diag(S))
    Lref = np.linalg.cholesky(full)
    got = np.nan_to_num(si.view(F, n), nan=0.0)
    assert np.allclose(got if uplo == "L" else got.T, Lref, rtol=1e-13, atol=1e-14)
    info, R, G = oracle.potrf_resid(uplo, n, A, n + 2, F, n + 2)
    assert info == 0 and np.all(np.abs(R) <= (n + 1) * oracle.U64 * G)
    # the residual routine against a dense evaluation, and at sampled entries
    Ld = np.tril(got if uplo == "L" else got.T).astype(np.longdouble)
    dense = full.astype(np.longdouble) - Ld @ Ld.T
    mask = oracle.triangle_mask(uplo, n)
    assert np.allclose(R[mask], dense.T[mask], rtol=0, atol=1e-16 * n)
    ii, jj = np.nonzero(mask.T)       # (row, col) pairs of the triangle
    sel = rng.choice(ii.size, 200, replace=False)
    info, Rs, Gs = oracle.potrf_resid(uplo, n, A, n + 2, F, n + 2, ii[sel], jj[sel])
    assert info == 0 and np.array_equal(Rs, R[jj[sel], ii[sel]]) and np.array_equal(Gs, G[jj[sel], ii[sel]])
    # a perturbed factor is caught
    Fbad = F.copy()
    Fbad[n // 3, n // 3] *= 1 + 1e-10
    _, R2, G2 = oracle.potrf_resid(uplo, n, A, n + 2, Fbad, n + 2)
    assert np.any(np.abs(R2) > 4 * n * oracle.U64 * G2)


def test_closed_forms_and_failure_reporting():
    A = np.array([[9.0]])
    assert oracle.potrf("L", 1, A, 1) == 0 and A[0, 0] == 3.0
    # [[4, 2], [2, 5]] = [[2, 0], [1, 2]] [[2, 1], [0, 2]]
    A = np.array([[4.0, 2.0], [np.nan, 5.0]])       # (col, row): lower triangle stored
    assert oracle.potrf("L", 2, A, 2) == 0
    assert A[0, 0] == 2.0 and A[0, 1] == 1.0 and A[1, 1] == 2.0 and np.isnan(A[1, 0])
    D = np.diag([4.0, 9.0, 16.0])
    assert oracle.potrf("U", 3, D, 3) == 0 and np.array_equal(np.diag(D), [2.0, 3.0, 4.0])
    # leading minor of order 3 is not positive definite: info = 3, columns 1-2 already factored
    M = np.array([[4.0, 2.0, 2.0], [2.0, 5.0, 3.0], [2.0, 3.0, 2.0]])      # 2 - 1 - 1 = 0 at the third pivot
    A = np.ascontiguousarray(M.T)
    assert oracle.potrf("L", 3, A, 3) == 3
    assert A[0, 0] == 2.0 and A[1, 1] == 2.0
    assert oracle.potrf("L", 0, None, 1) == 0
    assert oracle.potrf("X", 2, A, 3) == -1 and oracle.potrf("L", -1, A, 3) == -2
    assert oracle.potrf("L", 2, None, 3) == -3 and oracle.potrf("L", 3, A, 2) == -4
