"""Pins for the symmetric rank-k oracle: int64 products, exact rationals on tiny
shapes, symmetry between the two triangles, the untouched other triangle, scalar
paths and argument errors."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs as si


def opA(A, trans, n, k):
    r = n if trans == "N" else k
    V = si.view(A, r)
    return V if trans == "N" else V.T     # n x k


def make(rng, trans, n, k, pad=(0, 0), dtype=np.float64, kind="uniform", R=8):
    ra, ca = (n, k) if trans == "N" else (k, n)
    lda, ldc = max(ra, 1) + pad[0], max(n, 1) + pad[1]
    gen = (lambda r, c, ld: si.uniform(rng, r, c, ld, dtype)) if kind == "uniform" else \
        (lambda r, c, ld: si.integers(rng, r, c, ld, dtype, R=R))
    return gen(ra, ca, lda), lda, gen(n, n, ldc), ldc


@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("uplo,trans", list(itertools.product("LU", "NT")))
def test_integer_inputs_bit_exact_and_other_triangle_untouched(dtype, R, uplo, trans):
    rng = si.rng_for(95, 1)
    n, k = 37, 53
    mask = oracle.triangle_mask(uplo, n)
    for alpha, beta in [(1, 0), (-1, 1), (2, -1), (0, 2), (1, 1)]:
        A, lda, C, ldc = make(rng, trans, n, k, (3, 2), dtype, "int", R)
        a = opA(A, trans, n, k).astype(np.int64)
        want = alpha * (a @ a.T) + beta * si.view(C, n).astype(np.int64)     # (row, col)
        out = C.copy()
        assert oracle.syrk_work(uplo, trans, n, k, float(alpha), A, lda, float(beta), out, ldc) == 0
        got = out[:, :n]                                                       # (col, row)
        assert np.array_equal(got[mask], want.T[mask].astype(dtype))
        assert np.array_equal(got[~mask], C[:, :n][~mask])                     # other triangle untouched
        assert np.all(np.isnan(out[:, n:]))                                    # padding rows untouched
        info, Cref, G = oracle.syrk_ext(uplo, trans, n, k, float(alpha), A, lda, float(beta), C, ldc)
        assert info == 0 and np.array_equal(Cref[mask], want.T[mask].astype(Cref.dtype))
        assert not Cref[~mask].any() and not G[~mask].any()


def test_tiny_shapes_against_exact_rationals():
    rng = si.rng_for(95, 2)
    for n, k, uplo, trans in itertools.product([0, 1, 2, 3, 5], [0, 1, 2, 4], "LU", "NT"):
        A, lda, C, ldc = make(rng, trans, n, k, (1, 2))
        alpha, beta = 1.5, -0.5
        info, Cref, G = oracle.syrk_ext(uplo, trans, n, k, alpha, A, lda, beta, C, ldc)
        assert info == 0
        W = C.copy()
        assert oracle.syrk_work(uplo, trans, n, k, alpha, A, lda, beta, W, ldc) == 0
        a = opA(A, trans, n, k)
        for i in range(n):
            for j in range(n):
                if not ((i >= j) if uplo == "L" else (i <= j)):
                    assert W[j, i] == C[j, i]
                    continue
                ex = Fraction(alpha) * sum((Fraction(float(a[i, p])) * Fraction(float(a[j, p])) for p in range(k)),
                                           Fraction(0)) + Fraction(beta) * Fraction(float(C[j, i]))
                g = Fraction(float(G[j, i]))
                assert abs(Fraction(*Cref[j, i].as_integer_ratio()) - ex) <= Fraction(oracle.U64) / 256 * g + Fraction(1, 2 ** 1070)
                assert abs(Fraction(float(W[j, i])) - ex) <= Fraction(oracle.U64) * (k + 3) * g + Fraction(1, 2 ** 1070)


def test_lower_and_upper_are_transposes_of_each_other():
    rng = si.rng_for(95, 3)
    n, k = 41, 60
    A, lda, C, ldc = make(rng, "N", n, k)
    Csym = C.copy()
    Csym[:, :n] = (C[:, :n] + C[:, :n].T) / 2      # symmetric start
    L, U = Csym.copy(), Csym.copy()
    oracle.syrk_work("L", "N", n, k, 1.5, A, lda, -0.5, L, ldc)
    oracle.syrk_work("U", "N", n, k, 1.5, A, lda, -0.5, U, ldc)
    mask = oracle.triangle_mask("L", n)
    assert np.array_equal(L[:, :n][mask], U[:, :n].T[mask])     # a_i . a_j summed in the same order
    # and both agree with the general product oracle on their triangle
    At = np.ascontiguousarray(A)
    G_full = Csym.copy()
    oracle.gemm_work("N", "T", n, n, k, 1.5, A, lda, At, lda, -0.5, G_full, ldc)
    assert np.array_equal(L[:, :n][mask], G_full[:, :n][mask])


def test_scalar_paths_and_errors():
    n, k = 6, 4
    C0 = np.arange(36, dtype=np.float64).reshape(6, 6) + 1
    nanA = np.full((k, n), np.nan)
    C = C0.copy()
    assert oracle.syrk_work("L", "N", n, k, 0.0, nanA, n, 2.0, C, n) == 0      # alpha == 0: A not read
    m = oracle.triangle_mask("L", n)
    assert np.array_equal(C[m], 2 * C0[m]) and np.array_equal(C[~m], C0[~m])
    C = np.full((n, n), np.nan)
    A = np.ones((k, n))
    assert oracle.syrk_work("U", "N", n, k, 1.0, A, n, 0.0, C, n) == 0          # beta == 0 overwrites NaN
    mu = oracle.triangle_mask("U", n)
    assert np.array_equal(C[mu], np.full(mu.sum(), float(k))) and np.all(np.isnan(C[~mu]))
    C = C0.copy()
    assert oracle.syrk_work("L", "N", n, 0, 1.0, A, n, 1.0, C, n) == 0 and np.array_equal(C, C0)
    s = oracle.syrk_work
    assert s("X", "N", n, k, 1.0, A, n, 0.0, C, n) == -1
    assert s("L", "Q", n, k, 1.0, A, n, 0.0, C, n) == -2
    assert s("L", "N", -1, k, 1.0, A, n, 0.0, C, n) == -3
    assert s("L", "N", n, -1, 1.0, A, n, 0.0, C, n) == -4
    assert s("L", "N", n, k, 1.0, None, n, 0.0, C, n) == -6
    assert s("L", "N", n, k, 1.0, A, n - 1, 0.0, C, n) == -7
    assert s("L", "T", n, k, 1.0, A, k - 1, 0.0, C, n) == -7
    assert s("L", "N", n, k, 1.0, A, n, 0.0, None, n) == -9
    assert s("L", "N", n, k, 1.0, A, n, 0.0, C, n - 1) == -10
