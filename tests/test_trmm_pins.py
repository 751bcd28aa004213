"""Pins for the triangular-product oracle: int64 products, exact rationals on
tiny shapes, the general-product oracle on a densified triangle, the solve
oracle as its inverse, closed forms, scalar paths and error codes."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs as si

FLAGS = list(itertools.product("LR", "LU", "NT", "NU"))


def dense_op_T(A, dim, uplo, trans, diag):
    S = np.nan_to_num(si.view(A, dim).copy(), nan=0.0)
    T = np.tril(S) if uplo == "L" else np.triu(S)
    if diag == "U":
        np.fill_diagonal(T, 1.0)
    return T.T if trans == "T" else T


@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_integer_inputs_bit_exact(dtype, R, side, uplo, trans, diag):
    rng = si.rng_for(130, 1)
    m, n = 37, 29
    dim = m if side == "L" else n
    A = si.integers(rng, dim, dim, dim + 2, dtype, R)
    si._mask_triangle(A, dim, uplo, diag == "U", np.nan)
    B = si.integers(rng, m, n, m + 3, dtype, R)
    T = dense_op_T(A, dim, uplo, trans, diag).astype(np.int64)
    Bi = si.view(B, m).astype(np.int64)
    for alpha in (1, -2, 0):
        want = alpha * (T @ Bi if side == "L" else Bi @ T)
        out = B.copy()
        assert oracle.trmm_work(side, uplo, trans, diag, m, n, float(alpha), A, dim + 2, out, m + 3) == 0
        assert np.array_equal(si.view(out, m), want.astype(dtype)) and np.all(np.isnan(out[:, m:]))
        info, E, G = oracle.trmm_ext(side, uplo, trans, diag, m, n, float(alpha), A, dim + 2, B, m + 3)
        assert info == 0 and np.array_equal(E.T, want.astype(E.dtype))


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_tiny_shapes_against_exact_rationals(side, uplo, trans, diag):
    rng = si.rng_for(130, 2)
    for m, n in [(1, 1), (2, 3), (5, 4), (0, 3), (3, 0)]:
        dim = m if side == "L" else n
        A = si.triangular(rng, dim, dim + 1, np.float64, uplo, diag == "U")
        B = si.uniform(rng, m, n, m + 2)
        info, E, G = oracle.trmm_ext(side, uplo, trans, diag, m, n, 1.5, A, dim + 1, B, m + 2)
        W = B.copy()
        assert info == 0 and oracle.trmm_work(side, uplo, trans, diag, m, n, 1.5, A, dim + 1, W, m + 2) == 0
        T = dense_op_T(A, dim, uplo, trans, diag)
        Fr = lambda M: [[Fraction(float(v)) for v in row] for row in M]
        Tq, Bq = Fr(T), Fr(si.view(B, m))
        for i in range(m):
            for j in range(n):
                terms = [Tq[i][c] * Bq[c][j] for c in range(m)] if side == "L" else [Bq[i][c] * Tq[c][j] for c in range(n)]
                ex = Fraction(3, 2) * sum(terms, Fraction(0))
                g = Fraction(float(G[j, i]))
                assert abs(Fraction(*E[j, i].as_integer_ratio()) - ex) <= Fraction(oracle.U64) / 256 * g
                assert abs(Fraction(float(W[j, i])) - ex) <= Fraction(oracle.U64) * (dim + 2) * g


@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_equals_general_product_on_the_densified_triangle_and_inverts_the_solve(side, uplo, trans, diag):
    rng = si.rng_for(130, 3)
    m, n = 45, 38
    dim = m if side == "L" else n
    A = si.triangular(rng, dim, dim + 2, np.float64, uplo, diag == "U")
    B = si.uniform(rng, m, n, m + 1)
    info, E, G = oracle.trmm_ext(side, uplo, trans, diag, m, n, -0.75, A, dim + 2, B, m + 1)
    assert info == 0
    Td = np.ascontiguousarray(dense_op_T(A, dim, uplo, "N", diag).T)        # stored form, zeros filled in, ld = dim
    C0 = np.zeros((n, m))
    if side == "L":
        info, Cref, G2 = oracle.gemm_ext(trans, "N", m, n, m, -0.75, Td, dim, B, m + 1, 0.0, C0, m)
    else:
        info, Cref, G2 = oracle.gemm_ext("N", trans, m, n, n, -0.75, B, m + 1, Td, dim, 0.0, C0, m)
    assert info == 0 and np.array_equal(E, Cref) and np.array_equal(G, G2)
    # solving with the product as right-hand side returns B
    P = si.constant(m, n, m, np.float64)
    P[:, :m] = E.astype(np.float64)
    assert oracle.trsm_work(side, uplo, trans, diag, m, n, 1.0 / -0.75, A, dim + 2, P, m) == 0
    assert np.allclose(P, B[:, :m], rtol=1e-12, atol=1e-13)


def test_scalar_paths_and_errors():
    m, n = 6, 4
    B = np.full((n, m + 1), np.nan)
    assert oracle.trmm_work("L", "L", "N", "N", m, n, 0.0, None, m, B, m + 1) == 0     # alpha == 0: zeros, T unread
    assert np.all(B[:, :m] == 0) and np.all(np.isnan(B[:, m:]))
    A, Bm = np.eye(m), np.ones((n, m))
    t = oracle.trmm_work
    assert t("X", "L", "N", "N", m, n, 1.0, A, m, Bm, m) == -1
    assert t("L", "X", "N", "N", m, n, 1.0, A, m, Bm, m) == -2
    assert t("L", "L", "X", "N", m, n, 1.0, A, m, Bm, m) == -3
    assert t("L", "L", "N", "X", m, n, 1.0, A, m, Bm, m) == -4
    assert t("L", "L", "N", "N", -1, n, 1.0, A, m, Bm, m) == -5
    assert t("L", "L", "N", "N", m, -1, 1.0, A, m, Bm, m) == -6
    assert t("L", "L", "N", "N", m, n, 1.0, None, m, Bm, m) == -8
    assert t("L", "L", "N", "N", m, n, 1.0, A, m - 1, Bm, m) == -9
    assert t("R", "L", "N", "N", m, n, 1.0, A, n - 1, Bm, m) == -9
    assert t("L", "L", "N", "N", m, n, 1.0, A, m, None, m) == -10
    assert t("L", "L", "N", "N", m, n, 1.0, A, m, Bm, m - 1) == -11
