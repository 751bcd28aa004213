"""Pins for the symmetric-product and rank-2k oracles: int64 products, exact
rationals on tiny shapes, the general-product oracle on densified operands, the
rank-k oracle as the special case B = A / 2, untouched parts, scalars, errors."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs as si


def sym_dense(A, dim, uplo):
    S = np.nan_to_num(si.view(A, dim).copy(), nan=0.0)
    T = np.tril(S) if uplo == "L" else np.triu(S)
    return T + T.T - np.diag(np.diag(T))


def make_sym(rng, dim, ld, uplo, dtype=np.float64, kind="uniform", R=8):
    A = si.uniform(rng, dim, dim, ld, dtype) if kind == "uniform" else si.integers(rng, dim, dim, ld, dtype, R)
    return si._mask_triangle(A, dim, uplo, False, np.nan)


@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("side,uplo", list(itertools.product("LR", "LU")))
def test_symm_integer_bit_exact(dtype, R, side, uplo):
    rng = si.rng_for(200, 1)
    m, n = 37, 29
    dim = m if side == "L" else n
    A = make_sym(rng, dim, dim + 2, uplo, dtype, "int", R)
    B, C = si.integers(rng, m, n, m + 1, dtype, R), si.integers(rng, m, n, m + 3, dtype, R)
    S, Bi, Ci = sym_dense(A, dim, uplo).astype(np.int64), si.view(B, m).astype(np.int64), si.view(C, m).astype(np.int64)
    for alpha, beta in [(1, 0), (-2, 1), (0, 3)]:
        want = alpha * (S @ Bi if side == "L" else Bi @ S) + beta * Ci
        out = C.copy()
        assert oracle.symm_work(side, uplo, m, n, float(alpha), A, dim + 2, B, m + 1, float(beta), out, m + 3) == 0
        assert np.array_equal(si.view(out, m), want.astype(dtype)) and np.all(np.isnan(out[:, m:]))
        info, E, G = oracle.symm_ext(side, uplo, m, n, float(alpha), A, dim + 2, B, m + 1, float(beta), C, m + 3)
        assert info == 0 and np.array_equal(E.T, want.astype(E.dtype))


@pytest.mark.parametrize("side,uplo", list(itertools.product("LR", "LU")))
def test_symm_equals_general_product_on_densified_matrix_and_exact_rationals(side, uplo):
    rng = si.rng_for(200, 2)
    m, n = 23, 17
    dim = m if side == "L" else n
    A = make_sym(rng, dim, dim + 1, uplo)
    B, C = si.uniform(rng, m, n, m + 2), si.uniform(rng, m, n, m)
    info, E, G = oracle.symm_ext(side, uplo, m, n, 1.5, A, dim + 1, B, m + 2, -0.5, C, m)
    Sd = np.ascontiguousarray(sym_dense(A, dim, uplo).T)
    if side == "L":
        info2, E2, G2 = oracle.gemm_ext("N", "N", m, n, m, 1.5, Sd, dim, B, m + 2, -0.5, C, m)
    else:
        info2, E2, G2 = oracle.gemm_ext("N", "N", m, n, n, 1.5, B, m + 2, Sd, dim, -0.5, C, m)
    assert info == 0 and info2 == 0 and np.array_equal(E, E2) and np.array_equal(G, G2)
    # three entries against exact rational arithmetic
    S = sym_dense(A, dim, uplo)
    for i, j in [(0, 0), (m - 1, n - 1), (m // 2, n // 3)]:
        terms = [Fraction(float(S[i, c])) * Fraction(float(B[j, c])) for c in range(m)] if side == "L" else \
                [Fraction(float(B[c, i])) * Fraction(float(S[c, j])) for c in range(n)]
        ex = Fraction(3, 2) * sum(terms, Fraction(0)) - Fraction(1, 2) * Fraction(float(C[j, i]))
        assert abs(Fraction(*E[j, i].as_integer_ratio()) - ex) <= Fraction(oracle.U64) / 256 * Fraction(float(G[j, i]))


@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("uplo,trans", list(itertools.product("LU", "NT")))
def test_syr2k_integer_bit_exact_and_other_triangle_untouched(dtype, R, uplo, trans):
    rng = si.rng_for(200, 3)
    n, k = 31, 44
    ra, ca = (n, k) if trans == "N" else (k, n)
    A, B = si.integers(rng, ra, ca, ra + 1, dtype, R), si.integers(rng, ra, ca, ra + 2, dtype, R)
    C = si.integers(rng, n, n, n + 3, dtype, R)
    a = (si.view(A, ra) if trans == "N" else si.view(A, ra).T).astype(np.int64)
    b = (si.view(B, ra) if trans == "N" else si.view(B, ra).T).astype(np.int64)
    mask = oracle.triangle_mask(uplo, n)
    for alpha, beta in [(1, 0), (-1, 2), (0, -1)]:
        want = alpha * (a @ b.T + b @ a.T) + beta * si.view(C, n).astype(np.int64)
        out = C.copy()
        assert oracle.syr2k_work(uplo, trans, n, k, float(alpha), A, ra + 1, B, ra + 2, float(beta), out, n + 3) == 0
        assert np.array_equal(out[:, :n][mask], want.T[mask].astype(dtype))
        assert np.array_equal(out[:, :n][~mask], C[:, :n][~mask]) and np.all(np.isnan(out[:, n:]))


def test_syr2k_reduces_to_the_rank_k_update_and_to_two_general_products():
    rng = si.rng_for(200, 4)
    n, k = 27, 35
    A, B, C = si.uniform(rng, n, k, n + 1), si.uniform(rng, n, k, n + 1), si.uniform(rng, n, n, n)
    # B = A: alpha (A A^T + A A^T) = 2 alpha A A^T, exactly (doubling is exact)
    info, E, G = oracle.syr2k_ext("L", "N", n, k, 0.75, A, n + 1, A, n + 1, -0.5, C, n)
    info2, E2, G2 = oracle.syrk_ext("L", "N", n, k, 1.5, A, n + 1, -0.5, C, n)
    mask = oracle.triangle_mask("L", n)
    assert info == 0 and info2 == 0 and np.allclose(E[mask], E2[mask], rtol=1e-16, atol=1e-18)
    # general case: the two products accumulated by the general-product oracle
    info, E, G = oracle.syr2k_ext("U", "N", n, k, 1.5, A, n + 1, B, n + 1, 0.0, C, n)
    Z = np.zeros((n, n))
    _, P1, _ = oracle.gemm_ext("N", "T", n, n, k, 1.5, A, n + 1, B, n + 1, 0.0, Z, n)
    _, P2, _ = oracle.gemm_ext("N", "T", n, n, k, 1.5, B, n + 1, A, n + 1, 0.0, Z, n)
    mu = oracle.triangle_mask("U", n)
    assert np.allclose(E[mu], (P1 + P2)[mu], rtol=1e-16, atol=1e-18)
    assert not E[~mu].any()


def test_scalar_paths_and_errors():
    n, k = 5, 3
    A = np.ones((k, n)); C = np.full((n, n), np.nan)
    assert oracle.syr2k_work("L", "N", n, k, 1.0, A, n, A, n, 0.0, C, n) == 0       # beta == 0 overwrites NaN
    m = oracle.triangle_mask("L", n)
    assert np.all(C[m] == 2.0 * k) and np.all(np.isnan(C[~m]))
    C2 = np.arange(25, dtype=np.float64).reshape(5, 5)
    keep = C2.copy()
    assert oracle.syr2k_work("U", "T", n, 0, 1.0, None, 1, None, 1, 1.0, C2, n) == 0 and np.array_equal(C2, keep)
    s2 = oracle.syr2k_work
    assert s2("X", "N", n, k, 1.0, A, n, A, n, 0.0, C, n) == -1 and s2("L", "X", n, k, 1.0, A, n, A, n, 0.0, C, n) == -2
    assert s2("L", "N", -1, k, 1.0, A, n, A, n, 0.0, C, n) == -3 and s2("L", "N", n, -1, 1.0, A, n, A, n, 0.0, C, n) == -4
    assert s2("L", "N", n, k, 1.0, None, n, A, n, 0.0, C, n) == -6 and s2("L", "N", n, k, 1.0, A, n - 1, A, n, 0.0, C, n) == -7
    assert s2("L", "N", n, k, 1.0, A, n, None, n, 0.0, C, n) == -8 and s2("L", "T", n, k, 1.0, A, k, A, k - 1, 0.0, C, n) == -9
    assert s2("L", "N", n, k, 1.0, A, n, A, n, 0.0, None, n) == -11 and s2("L", "N", n, k, 1.0, A, n, A, n, 0.0, C, n - 1) == -12
    S = np.eye(4); B = np.ones((3, 4)); Cm = np.full((3, 4), np.nan)
    assert oracle.symm_work("L", "U", 4, 3, 2.0, S, 4, B, 4, 0.0, Cm, 4) == 0 and np.all(Cm == 2.0)
    sm = oracle.symm_work
    assert sm("X", "L", 4, 3, 1.0, S, 4, B, 4, 0.0, Cm, 4) == -1 and sm("L", "X", 4, 3, 1.0, S, 4, B, 4, 0.0, Cm, 4) == -2
    assert sm("L", "L", -1, 3, 1.0, S, 4, B, 4, 0.0, Cm, 4) == -3 and sm("L", "L", 4, -1, 1.0, S, 4, B, 4, 0.0, Cm, 4) == -4
    assert sm("L", "L", 4, 3, 1.0, None, 4, B, 4, 0.0, Cm, 4) == -6 and sm("L", "L", 4, 3, 1.0, S, 3, B, 4, 0.0, Cm, 4) == -7
    assert sm("R", "L", 4, 3, 1.0, S, 2, B, 4, 0.0, Cm, 4) == -7 and sm("L", "L", 4, 3, 1.0, S, 4, None, 4, 0.0, Cm, 4) == -8
    assert sm("L", "L", 4, 3, 1.0, S, 4, B, 3, 0.0, Cm, 4) == -9 and sm("L", "L", 4, 3, 1.0, S, 4, B, 4, 0.0, None, 4) == -11
    assert sm("L", "L", 4, 3, 1.0, S, 4, B, 4, 0.0, Cm, 3) == -12
