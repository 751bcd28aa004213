"""Pins of the LU oracle (CPU only): factorisations known exactly, a library's partial-pivoting LU, exact
rational elimination on tiny matrices, the tie rule, singular columns, rectangular shapes, and the residual
routine against a dense evaluation.  Planted mistakes must fail."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.linalg

import oracle
import synth_inputs as si
from lu_util import check_valid, perm_of, planted_lu, unpack


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("m,n", [(1, 1), (7, 7), (64, 64), (200, 131), (131, 200), (300, 300)])
def test_planted_factorisation_is_recovered_exactly(dtype, m, n):
    rng = si.rng_for(300, m * 1000 + n)
    A, L, U, perm = planted_lu(rng, m, n, dtype, ld=m + 3)
    F = A.copy()
    info, ipiv = oracle.getrf(m, n, F, m + 3)
    assert info == 0
    Lg, Ug = unpack(F, m, n)
    # the first min(m, n) rows of P A are fixed by the pivots; the order of the rows below them is whatever
    # the interchanges left, so those rows of L are compared through the row of A they came from
    src, where = perm_of(ipiv, m), np.argsort(perm)          # where[a]: planted position of row a of A
    assert np.array_equal(src[:min(m, n)], perm[:min(m, n)])
    assert np.array_equal(Lg, L[where[src], :]) and np.array_equal(Ug, U)
    assert np.all(np.isnan(F[:, m:]))                       # padding rows untouched
    # and the residual routine agrees that it is exact
    rinfo, R, G = oracle.getrf_resid(m, n, A, m + 3, F, m + 3, ipiv)
    assert rinfo == 0 and not R.any() and np.all(G >= 0)


@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-11), (np.float32, 2e-3)])
@pytest.mark.parametrize("m,n", [(50, 50), (257, 257), (300, 120), (120, 300)])
def test_against_a_library_factorisation(dtype, tol, m, n):
    rng = si.rng_for(301, m + n)
    A = si.uniform(rng, m, n, m, dtype)
    F = A.copy()
    info, ipiv = oracle.getrf(m, n, F, m)
    assert info == 0
    lu, piv = scipy.linalg.lu_factor(A.T.astype(dtype), check_finite=False) if m == n else (None, None)
    if m == n:
        assert np.array_equal(ipiv - 1, piv)
        assert np.allclose(F.T, lu, rtol=tol, atol=tol)
    else:
        P, Ls, Us = scipy.linalg.lu(A.T.astype(np.float64))                   # A = P L U
        Lg, Ug = unpack(F, m, n)
        src = perm_of(ipiv, m)
        assert np.allclose(A.T.astype(np.float64)[src, :], Lg @ Ug, rtol=tol, atol=tol)
        assert np.allclose(Lg, Ls, rtol=tol, atol=tol) and np.allclose(Ug, Us, rtol=tol, atol=tol)
    check_valid(m, n, A, m, F, m, ipiv, oracle.U64 if dtype == np.float64 else oracle.U32)


def _exact_lu(rows):
    """Gaussian elimination with partial pivoting (first largest candidate) in exact rational arithmetic."""
    A = [[Fraction(x) for x in r] for r in rows]
    m, n = len(A), len(A[0])
    piv = []
    for j in range(min(m, n)):
        p = max(range(j, m), key=lambda i: (abs(A[i][j]), -i))
        piv.append(p + 1)
        if A[p][j] != 0:
            A[j], A[p] = A[p], A[j]
            for i in range(j + 1, m):
                A[i][j] /= A[j][j]
        for i in range(j + 1, m):
            for c in range(j + 1, n):
                A[i][c] -= A[i][j] * A[j][c]
    return A, piv


def test_tiny_matrices_against_exact_rational_elimination():
    rng = si.rng_for(302, 0)
    for m, n in [(1, 1), (2, 2), (3, 3), (4, 6), (6, 4), (5, 5), (8, 8)]:
        for _ in range(20):
            rows = rng.integers(-9, 10, size=(m, n))
            want, piv = _exact_lu(rows.tolist())
            A = np.ascontiguousarray(rows.T.astype(np.float64))
            info, ipiv = oracle.getrf(m, n, A, m)
            # ties between candidates are decided alike (first largest); magnitudes here are exact small integers
            # only in the first column, so compare pivots where the exact candidates are not tied within rounding
            got = A.T
            exact = np.array([[float(x) for x in r] for r in want])
            if list(ipiv) == piv:
                assert np.allclose(got, exact, rtol=1e-12, atol=1e-12)
            zero_pivot = next((j + 1 for j in range(min(m, n)) if want[j][j] == 0), 0)
            if list(ipiv) == piv and all(abs(float(want[j][j])) > 1e-9 or want[j][j] == 0 for j in range(min(m, n))):
                assert info == zero_pivot
    # the first column is decided on exact integers: the pivot is the first of the largest
    A = np.array([[1.0, -3.0, 3.0, 2.0]])                  # one column, m = 4 (layout (col, row))
    info, ipiv = oracle.getrf(4, 1, A, 4)
    assert info == 0 and list(ipiv) == [2] and np.array_equal(A[0], [-3.0, -1.0 / 3.0, -1.0, -2.0 / 3.0])


def test_tie_rule_takes_the_first_of_equal_candidates():
    # column (2, -2, 2): row 1 stays; after the step the second column decides between equal candidates again
    A = np.array([[2.0, -2.0, 2.0], [1.0, 3.0, 5.0], [0.0, 1.0, 4.0]])        # columns of the matrix
    F = A.copy()
    info, ipiv = oracle.getrf(3, 3, F, 3)
    assert info == 0 and ipiv[0] == 1
    # second column after elimination: rows 2, 3 hold 3 + 1 = 4 and 5 - 1 = 4: tie, the first (row 2) wins
    assert ipiv[1] == 2 and ipiv[2] == 3
    assert np.array_equal(F[0], [2.0, -1.0, 1.0]) and np.array_equal(F[1], [1.0, 4.0, 1.0])


def test_zero_pivot_is_reported_and_the_elimination_goes_on():
    A = np.array([[0.0, 0.0], [1.0, 2.0]])                 # matrix [[0, 1], [0, 2]]
    F = A.copy()
    info, ipiv = oracle.getrf(2, 2, F, 2)
    assert info == 1 and list(ipiv) == [1, 2] and np.array_equal(F, A)
    # a zero column in the middle: info names it, later columns are still eliminated
    rng = si.rng_for(303, 0)
    M = rng.uniform(-1, 1, size=(6, 6))
    M[:, 2] = 0.5 * M[:, 0] - 2.0 * M[:, 1]                # rank deficient: column 3 depends on columns 1, 2
    F = np.ascontiguousarray(M.T)
    info, ipiv = oracle.getrf(6, 6, F, 6)
    L, U = unpack(F, 6, 6)
    assert abs(U[2, 2]) < 1e-14 and info in (0, 3)         # an exact zero only if the roundings cancel
    assert np.allclose(M[perm_of(ipiv, 6), :], L @ U, atol=1e-14)
    Z = np.zeros((3, 4))
    info, ipiv = oracle.getrf(4, 3, Z, 4)
    assert info == 1 and list(ipiv) == [1, 2, 3] and not Z.any()


def test_error_codes_and_empty_shapes():
    A = np.zeros((4, 5))
    ip = np.zeros(4, dtype=np.int32)
    L = oracle.lib()
    assert L.ref_dgetrf(-1, 4, A.ctypes.data, 5, ip.ctypes.data) == -1
    assert L.ref_dgetrf(5, -1, A.ctypes.data, 5, ip.ctypes.data) == -2
    assert L.ref_dgetrf(5, 4, None, 5, ip.ctypes.data) == -3
    assert L.ref_dgetrf(5, 4, A.ctypes.data, 4, ip.ctypes.data) == -4
    assert L.ref_dgetrf(5, 4, A.ctypes.data, 5, None) == -5
    assert L.ref_sgetrf(0, 4, None, 1, None) == 0 and L.ref_dgetrf(4, 0, None, 4, None) == 0


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_residual_routine_against_a_dense_evaluation(dtype):
    rng = si.rng_for(304, 0)
    m, n = 37, 29
    A = si.uniform(rng, m, n, m + 2, dtype)
    F = A.copy()
    info, ipiv = oracle.getrf(m, n, F, m + 2)
    assert info == 0
    rinfo, R, G = oracle.getrf_resid(m, n, A, m + 2, F, m + 2, ipiv)
    assert rinfo == 0
    L, U = unpack(F, m, n)
    wide = np.longdouble
    PA = A[:, :m].T.astype(wide)[perm_of(ipiv, m), :]
    Rd = PA - L.astype(wide) @ U.astype(wide)
    Gd = np.abs(L).astype(wide) @ np.abs(U).astype(wide)
    # both are sums of the same products in the wide type, in different orders
    wide_eps = float(np.finfo(R.dtype).eps)
    assert np.allclose(R.T.astype(np.float64), Rd.astype(np.float64), rtol=0, atol=32 * wide_eps * float(Gd.max()))
    assert float(np.abs(Rd).max()) > 10 * 32 * wide_eps * float(Gd.max())     # the comparison resolves the residual
    assert np.allclose(G.T.astype(np.float64), Gd.astype(np.float64), rtol=1e-12)
    # the sampled form returns the same numbers
    I, J = si.sample_indices(rng, m, n, 3, 3, 50)
    sinfo, Rs, Gs = oracle.getrf_resid(m, n, A, m + 2, F, m + 2, ipiv, I, J)
    assert sinfo == 0 and np.array_equal(Rs, R[J, I]) and np.array_equal(Gs, G[J, I])
    # an illegal interchange is refused
    bad = ipiv.copy()
    bad[3] = 2
    assert oracle.getrf_resid(m, n, A, m + 2, F, m + 2, bad)[0] == 7


def test_planted_mistakes_fail_the_validity_statement():
    rng = si.rng_for(305, 0)
    n = 60
    A = si.uniform(rng, n, n, n)
    F = A.copy()
    info, ipiv = oracle.getrf(n, n, F, n)
    check_valid(n, n, A, n, F, n, ipiv, oracle.U64)
    # interchanges not applied to the columns already factored (the multipliers stay behind)
    G2 = A.copy()
    _, ip2 = oracle.getrf(n, n, G2, n)
    j = int(np.argmax(ip2 - 1 != np.arange(n)) + 5)
    while ip2[j] - 1 == j:
        j += 1
    G2[:j, [j, ip2[j] - 1]] = G2[:j, [ip2[j] - 1, j]]       # undo interchange j on the columns to its left
    with pytest.raises(AssertionError):
        check_valid(n, n, A, n, G2, n, ip2, oracle.U64)
    # a wrong pivot choice (not the largest candidate) shows as a multiplier above one
    B = np.array([[1.0, 4.0], [2.0, 3.0]])                  # matrix [[1, 2], [4, 3]]: the pivot must be 4
    Fb = np.array([[1.0, 4.0], [2.0, -5.0]])                # elimination without the interchange
    with pytest.raises(AssertionError):
        check_valid(2, 2, B, 2, Fb, 2, np.array([1, 2]), oracle.U64)
    # one entry of U off by a few units in the last place of the largest term
    F3 = F.copy()
    F3[n - 1, n - 2] *= 1.0 + 1e-9
    with pytest.raises(AssertionError):
        check_valid(n, n, A, n, F3, n, ipiv, oracle.U64)
    # two interchanges swapped in the record
    ip4 = ipiv.copy()
    a = int(np.argmax(ipiv[:-1] != ipiv[1:]))
    ip4[a], ip4[a + 1] = max(ipiv[a + 1], a + 1), max(ipiv[a], a + 2)
    if not np.array_equal(ip4, ipiv):
        with pytest.raises(AssertionError):
            check_valid(n, n, A, n, F, n, ip4, oracle.U64)
