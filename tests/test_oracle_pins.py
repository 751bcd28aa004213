"""Pins for the CPU oracle: it is checked against things other than itself.

* exact rational arithmetic (fractions.Fraction) on every tiny shape,
* int64 matrix products on integer-valued inputs (bit-exact),
* closed forms (ones, identity, separable ramps, rank-1),
* the BLAS scalar paths (alpha = 0, beta = 0, k = 0, empty m or n),
* invariants (linearity, transpose identity, padding invariance),
* the textbook forward error bound  |fl(sum) - sum| <= gamma_k sum|a||b|,
* numpy's own float64/complex128 matmul as a third opinion.

The definition pinned is the sum of outer products of paper Sec. 2.1 with the
column-major BLAS scalars and transposes around it.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs as si

TRANS = ["N", "T"]


def stored(trans, rows_op, cols_op):
    return si.operand_shape(trans, rows_op, cols_op)


def make_operands(rng, ta, tb, m, n, k, pad=(0, 0, 0), dtype=np.float64, kind="uniform", R=8):
    ra, ca = stored(ta, m, k)
    rb, cb = stored(tb, k, n)
    lda, ldb, ldc = max(ra, 1) + pad[0], max(rb, 1) + pad[1], max(m, 1) + pad[2]
    if kind == "uniform":
        gen = lambda r, c, ld: si.uniform(rng, r, c, ld, dtype)
    elif kind == "normal":
        gen = lambda r, c, ld: si.normal(rng, r, c, ld, dtype)
    else:
        gen = lambda r, c, ld: si.integers(rng, r, c, ld, dtype, R=R)
    A, B, C = gen(ra, ca, lda), gen(rb, cb, ldb), gen(m, n, ldc)
    return A, lda, B, ldb, C, ldc


def op_view(X, trans, rows_op, cols_op):
    """op(X) as a (rows_op, cols_op) array."""
    r, _ = stored(trans, rows_op, cols_op)
    V = si.view(X, r)
    return V if trans in "Nn" else V.T


# --------------------------------------------------------------------------
# 1. exact rational brute force on every tiny shape
# --------------------------------------------------------------------------
def exact_gemm(ta, tb, m, n, k, alpha, A, B, beta, C):
    opA, opB, Cin = op_view(A, ta, m, k), op_view(B, tb, k, n), si.view(C, m)
    out = [[None] * n for _ in range(m)]
    mag = [[None] * n for _ in range(m)]
    fa, fb = Fraction(float(alpha)), Fraction(float(beta))
    for i in range(m):
        for j in range(n):
            s, g = Fraction(0), Fraction(0)
            for p in range(k):
                t = Fraction(float(opA[i, p])) * Fraction(float(opB[p, j]))
                s += t
                g += abs(t)
            r, gg = fa * s, abs(fa) * g
            if beta != 0:
                c = Fraction(float(Cin[i, j]))
                r += fb * c
                gg += abs(fb) * abs(c)
            out[i][j], mag[i][j] = r, gg
    return out, mag


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_tiny_shapes_against_exact_rationals(dtype):
    rng = si.rng_for(90, 1)
    u = oracle.U64 if dtype == np.float64 else oracle.U32
    dims = [0, 1, 2, 3, 5]
    ncase = 0
    for (m, n, k), ta, tb, pad in itertools.product(
            itertools.product(dims, dims, dims), TRANS, TRANS, [(0, 0, 0), (3, 1, 2)]):
        alpha, beta = [(1.0, 0.0), (1.5, -0.5), (-1.0, 1.0), (0.0, 2.0)][ncase % 4]
        ncase += 1
        A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad, dtype)
        want, mag = exact_gemm(ta, tb, m, n, k, alpha, A, B, beta, C)
        info, Cref, G = oracle.gemm_ext(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc)
        assert info == 0
        Cw = C.copy()
        assert oracle.gemm_work(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, Cw, ldc) == 0
        # padding rows of C never touched
        assert np.all(np.isnan(Cw[:, m:]))
        for i in range(m):
            for j in range(n):
                ex, g = want[i][j], mag[i][j]
                # extended: error far below one working-precision ulp of G
                err_ext = abs(Fraction(float(Cref[j, i])) - ex) if dtype == np.float32 else \
                    abs(Fraction(*(Cref[j, i].as_integer_ratio())) - ex)
                assert err_ext <= Fraction(u) * Fraction(1, 256) * g + Fraction(1, 2 ** 1070)
                assert abs(Fraction(float(G[j, i])) - g) <= Fraction(u) * g * (k + 4)
                # working precision: standard bound gamma_{k+2} * G (<= (k+3) u G here)
                err_w = abs(Fraction(float(Cw[j, i])) - ex)
                assert err_w <= Fraction(u) * (k + 3) * g + Fraction(1, 2 ** 1070)
    assert ncase == 125 * 4 * 2


# --------------------------------------------------------------------------
# 2. integer-valued inputs: bit-exact against int64 arithmetic
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,R", [(np.float64, 1000), (np.float32, 8)])
@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
def test_integer_inputs_bit_exact(dtype, R, ta, tb):
    rng = si.rng_for(90, 2)
    m, n, k = 37, 29, 53
    for alpha, beta in [(1, 0), (-1, 1), (2, -1), (1, 2), (0, 2), (2, 0)]:
        A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, (2, 5, 1), dtype, "int", R)
        iA = op_view(A, ta, m, k).astype(np.int64)
        iB = op_view(B, tb, k, n).astype(np.int64)
        iC = si.view(C, m).astype(np.int64)
        want = alpha * (iA @ iB) + beta * iC
        assert np.abs(want).max() < (2 ** 53 if dtype == np.float64 else 2 ** 24)
        Cw = C.copy()
        assert oracle.gemm_work(ta, tb, m, n, k, float(alpha), A, lda, B, ldb, float(beta), Cw, ldc) == 0
        assert np.array_equal(si.view(Cw, m), want.astype(dtype))
        info, Cref, _ = oracle.gemm_ext(ta, tb, m, n, k, float(alpha), A, lda, B, ldb, float(beta), C, ldc)
        assert info == 0 and np.array_equal(Cref.T, want.astype(Cref.dtype))


# --------------------------------------------------------------------------
# 3. closed forms
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_all_ones_gives_k(dtype):
    m, n, k = 19, 23, 301
    A, B = si.constant(m, k, m + 1, dtype), si.constant(k, n, k + 3, dtype)
    C = si.constant(m, n, m, dtype, value=np.nan)
    assert oracle.gemm_work("N", "N", m, n, k, 1.0, A, m + 1, B, k + 3, 0.0, C, m) == 0
    assert np.array_equal(C, np.full((n, m), k, dtype=dtype))


@pytest.mark.parametrize("side", ["left", "right"])
def test_identity_factor(side):
    rng = si.rng_for(90, 3)
    m, n = 31, 17
    X = si.uniform(rng, m, n, m + 2)
    C0 = si.uniform(rng, m, n, m)
    for alpha, beta in [(1.0, 0.0), (1.0, 1.0), (2.0, -1.0)]:
        C = C0.copy()
        if side == "left":   # C = alpha I X + beta C
            E = si.identity(m)
            assert oracle.gemm_work("N", "N", m, n, m, alpha, E, m, X, m + 2, beta, C, m) == 0
        else:                # C = alpha X I + beta C
            E = si.identity(n)
            assert oracle.gemm_work("N", "T", m, n, n, alpha, X, m + 2, E, n, beta, C, m) == 0
        want = alpha * si.view(X, m) + (beta * si.view(C0, m) if beta != 0 else 0.0)
        assert np.array_equal(si.view(C, m), want)


def test_separable_ramp_closed_form():
    # A[i,p] = i+1, B[p,j] = j+1  =>  C[i,j] = k (i+1)(j+1), exact
    m, n, k = 40, 33, 77
    A = np.ascontiguousarray(np.tile(np.arange(1, m + 1, dtype=np.float64), (k, 1)))
    B = np.ascontiguousarray(np.repeat(np.arange(1, n + 1, dtype=np.float64)[:, None], k, axis=1))
    C = np.zeros((n, m))
    assert oracle.gemm_work("N", "N", m, n, k, 1.0, A, m, B, k, 0.0, C, m) == 0
    want = k * np.outer(np.arange(1, n + 1), np.arange(1, m + 1)).astype(np.float64)
    assert np.array_equal(C, want)
    # same data read through the transposed accessors
    At = np.ascontiguousarray(A.T)   # stored k x m: op = T
    Bt = np.ascontiguousarray(B.T)   # stored n x k: op = T
    C2 = np.zeros((n, m))
    assert oracle.gemm_work("T", "T", m, n, k, 1.0, At, k, Bt, n, 0.0, C2, m) == 0
    assert np.array_equal(C2, want)


def test_rank_one_update_per_element():
    rng = si.rng_for(90, 4)
    m, n = 13, 11
    a, b = si.uniform(rng, m, 1), si.uniform(rng, 1, n)
    C0 = si.uniform(rng, m, n)
    alpha, beta = 1.25, -0.75
    C = C0.copy()
    assert oracle.gemm_work("N", "N", m, n, 1, alpha, a, m, b, 1, beta, C, m) == 0
    for i in range(m):
        for j in range(n):
            want = alpha * (a[0, i] * b[j, 0]) + beta * C0[j, i]   # same 4 roundings
            assert C[j, i] == want


# --------------------------------------------------------------------------
# 4. scalar paths and quick returns
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_alpha_zero_does_not_read_a_b(dtype):
    rng = si.rng_for(90, 5)
    m, n, k = 9, 7, 5
    A = np.full((k, m), np.nan, dtype=dtype)
    B = np.full((n, k), np.nan, dtype=dtype)
    C0 = si.uniform(rng, m, n, m + 1, dtype)
    for beta in [0.0, 1.0, -1.0, 2.0, 0.5]:
        C = C0.copy()
        assert oracle.gemm_work("N", "N", m, n, k, 0.0, A, m, B, k, beta, C, m + 1) == 0
        assert np.array_equal(si.view(C, m), (dtype(beta) * si.view(C0, m)).astype(dtype))
        assert np.all(np.isnan(C[:, m:]))
        info, Cref, G = oracle.gemm_ext("N", "N", m, n, k, 0.0, A, m, B, k, beta, C0, m + 1)
        assert info == 0 and np.array_equal(Cref.T, beta * si.view(C0, m).astype(Cref.dtype))
    # null A/B are legal when alpha == 0
    C = C0.copy()
    assert oracle.gemm_work("N", "N", m, n, k, 0.0, None, m, None, k, 2.0, C, m + 1) == 0


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_beta_zero_overwrites_nan(dtype):
    rng = si.rng_for(90, 6)
    m, n, k = 9, 7, 5
    A, B = si.uniform(rng, m, k, m, dtype), si.uniform(rng, k, n, k, dtype)
    C = np.full((n, m), np.nan, dtype=dtype)
    assert oracle.gemm_work("N", "N", m, n, k, 1.0, A, m, B, k, 0.0, C, m) == 0
    assert np.all(np.isfinite(C))
    info, Cref, G = oracle.gemm_ext("N", "N", m, n, k, 1.0, A, m, B, k, 0.0,
                                    np.full((n, m), np.nan, dtype=dtype), m)
    assert info == 0 and np.all(np.isfinite(Cref)) and np.all(np.isfinite(G))
    # k == 0 behaves like alpha == 0
    C = np.full((n, m), np.nan, dtype=dtype)
    assert oracle.gemm_work("N", "N", m, n, 0, 1.0, A, m, B, 1, 0.0, C, m) == 0
    assert np.array_equal(C, np.zeros((n, m), dtype=dtype))


def test_empty_m_or_n_touches_nothing():
    C = np.full((4, 6), 7.0)
    A, B = np.ones((4, 6)), np.ones((4, 6))
    assert oracle.gemm_work("N", "N", 0, 4, 3, 1.0, A, 1, B, 3, 0.0, C, 6) == 0
    assert oracle.gemm_work("N", "N", 5, 0, 3, 1.0, A, 5, B, 3, 0.0, C, 6) == 0
    assert np.all(C == 7.0)


def test_argument_errors():
    A, B, C = np.ones((8, 8)), np.ones((8, 8)), np.ones((8, 8))
    g = lambda *a: oracle.gemm_work(*a)
    assert g("X", "N", 2, 2, 2, 1.0, A, 2, B, 2, 0.0, C, 2) == -1
    assert g("N", "Q", 2, 2, 2, 1.0, A, 2, B, 2, 0.0, C, 2) == -2
    assert g("N", "N", -1, 2, 2, 1.0, A, 2, B, 2, 0.0, C, 2) == -3
    assert g("N", "N", 2, -1, 2, 1.0, A, 2, B, 2, 0.0, C, 2) == -4
    assert g("N", "N", 2, 2, -1, 1.0, A, 2, B, 2, 0.0, C, 2) == -5
    assert g("N", "N", 2, 2, 2, 1.0, None, 2, B, 2, 0.0, C, 2) == -7
    assert g("N", "N", 3, 2, 2, 1.0, A, 2, B, 2, 0.0, C, 3) == -8    # lda < m
    assert g("T", "N", 3, 2, 4, 1.0, A, 3, B, 4, 0.0, C, 3) == -8    # lda < k for T
    assert g("N", "N", 2, 2, 2, 1.0, A, 2, None, 2, 0.0, C, 2) == -9
    assert g("N", "N", 2, 2, 3, 1.0, A, 2, B, 2, 0.0, C, 2) == -10   # ldb < k
    assert g("N", "T", 2, 3, 2, 1.0, A, 2, B, 2, 0.0, C, 2) == -10   # ldb < n for T
    assert g("N", "N", 2, 2, 2, 1.0, A, 2, B, 2, 0.0, None, 2) == -12
    assert g("N", "N", 3, 2, 2, 1.0, A, 3, B, 2, 0.0, C, 2) == -13
    assert g("N", "N", 0, 2, 2, 1.0, A, 0, B, 2, 0.0, C, 1) == -8    # ld must be >= 1
    assert g("n", "c", 2, 2, 2, 1.0, A, 2, B, 2, 0.0, C, 2) == 0     # lower case, C == T for reals


# --------------------------------------------------------------------------
# 5. invariants
# --------------------------------------------------------------------------
def test_linearity_on_integers():
    rng = si.rng_for(90, 7)
    m, n, k = 21, 18, 40
    A1, A2 = si.integers(rng, m, k, R=50), si.integers(rng, m, k, R=50)
    B = si.integers(rng, k, n, R=50)
    outs = []
    for A in (A1, A2, A1 + A2):
        C = np.zeros((n, m))
        assert oracle.gemm_work("N", "N", m, n, k, 3.0, A, m, B, k, 0.0, C, m) == 0
        outs.append(C)
    assert np.array_equal(outs[0] + outs[1], outs[2])


def test_transpose_identity():
    # (A B)^T = B^T A^T : computing the n x m product from the same buffers with
    # swapped roles must give the transposed result within twice the bound.
    rng = si.rng_for(90, 8)
    m, n, k = 26, 35, 64
    A, B = si.uniform(rng, m, k, m + 3), si.uniform(rng, k, n, k + 1)
    _, C1, G1 = oracle.gemm_ext("N", "N", m, n, k, 1.0, A, m + 3, B, k + 1, 0.0, np.zeros((n, m)), m)
    _, C2, _ = oracle.gemm_ext("T", "T", n, m, k, 1.0, B, k + 1, A, m + 3, 0.0, np.zeros((m, n)), n)
    assert np.all(np.abs(C1 - C2.T) <= 2 * 4 * k * oracle.U64 * G1)
    W1, W2 = np.zeros((n, m)), np.zeros((m, n))
    oracle.gemm_work("N", "N", m, n, k, 1.0, A, m + 3, B, k + 1, 0.0, W1, m)
    oracle.gemm_work("T", "T", n, m, k, 1.0, B, k + 1, A, m + 3, 0.0, W2, n)
    assert np.array_equal(W1, W2.T)   # same products, same order -> same bits


@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
def test_padding_invariance(ta, tb):
    m, n, k = 14, 9, 22
    res = []
    for pad in [(0, 0, 0), (1, 7, 5)]:
        rng = si.rng_for(90, 9)   # same draws for both paddings
        A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad)
        assert oracle.gemm_work(ta, tb, m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc) == 0
        res.append(si.view(C, m).copy())
    assert np.array_equal(res[0], res[1])


# --------------------------------------------------------------------------
# 6. error bound and library cross-check
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
def test_working_vs_extended_vs_numpy(dtype, ta, tb):
    rng = si.rng_for(90, 10)
    m, n, k = 70, 45, 200
    u = oracle.U64 if dtype == np.float64 else oracle.U32
    alpha, beta = 1.5, -0.5
    A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, (1, 2, 3), dtype)
    info, Cref, G = oracle.gemm_ext(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc)
    assert info == 0
    Cw = C.copy()
    assert oracle.gemm_work(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, Cw, ldc) == 0
    nviol, ratio = oracle.bound_violations(si.view(Cw, m).T, Cref, G, k, u)
    assert nviol == 0 and ratio < 0.5
    # numpy's matmul in float64 on the same operands is a third opinion
    ref_np = alpha * (op_view(A, ta, m, k).astype(np.float64) @ op_view(B, tb, k, n).astype(np.float64)) \
        + beta * si.view(C, m).astype(np.float64)
    tol = 4 * k * (oracle.U64 if dtype == np.float64 else 2.0 ** -40) * G.T.astype(np.float64)
    assert np.all(np.abs(ref_np - Cref.T.astype(np.float64)) <= tol)
    # G itself against numpy on absolute values
    G_np = abs(alpha) * (np.abs(op_view(A, ta, m, k)).astype(np.float64) @ np.abs(op_view(B, tb, k, n)).astype(np.float64)) \
        + abs(beta) * np.abs(si.view(C, m)).astype(np.float64)
    assert np.allclose(G.T.astype(np.float64), G_np, rtol=1e-6 if dtype == np.float32 else 1e-12)


def test_bound_checker_flags_planted_errors():
    rng = si.rng_for(90, 11)
    m, n, k = 12, 10, 30
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "N", m, n, k)
    _, Cref, G = oracle.gemm_ext("N", "N", m, n, k, 1.0, A, lda, B, ldb, 1.0, C, ldc)
    good = Cref.astype(np.float64)
    assert oracle.bound_violations(good, Cref, G, k, oracle.U64)[0] == 0
    bad = good.copy(); bad[3, 4] += 8 * k * oracle.U64 * float(G[3, 4])
    assert oracle.bound_violations(bad, Cref, G, k, oracle.U64)[0] == 1
    bad = good.copy(); bad[0, 0] = np.nan
    assert oracle.bound_violations(bad, Cref, G, k, oracle.U64)[0] == 1
    # a transposed operand, a dropped k-term and a sign error are all caught
    _, Ct, _ = oracle.gemm_ext("N", "N", m, n, k - 1, 1.0, A, lda, B, ldb, 1.0, C, ldc)
    assert oracle.bound_violations(Ct.astype(np.float64), Cref, G, k, oracle.U64)[0] > 0
    _, Cs, _ = oracle.gemm_ext("N", "N", m, n, k, 1.0, A, lda, B, ldb, -1.0, C, ldc)
    assert oracle.bound_violations(Cs.astype(np.float64), Cref, G, k, oracle.U64)[0] > 0


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_samples_match_full_reference(dtype):
    rng = si.rng_for(90, 12)
    m, n, k = 33, 27, 41
    for ta, tb in itertools.product(TRANS, TRANS):
        A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, (2, 0, 1), dtype)
        _, Cref, G = oracle.gemm_ext(ta, tb, m, n, k, -1.0, A, lda, B, ldb, 1.0, C, ldc)
        I, J = si.sample_indices(rng, m, n, 3, 3, 50)
        info, c, g = oracle.gemm_samples(ta, tb, m, n, k, -1.0, A, lda, B, ldb, 1.0, C, ldc, I, J)
        assert info == 0
        assert np.array_equal(c, Cref[J, I]) and np.array_equal(g, G[J, I])
    assert oracle.gemm_samples("N", "N", 3, 3, 3, 1.0, np.ones((3, 3), dtype), 3, np.ones((3, 3), dtype), 3,
                               0.0, np.ones((3, 3), dtype), 3, [3], [0])[0] == -14


def test_thread_count_does_not_change_bits():
    rng = si.rng_for(90, 13)
    m, n, k = 64, 48, 100
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "T", m, n, k)
    nt = oracle.num_threads()
    outs = []
    for t in (1, max(nt, 2)):
        oracle.set_num_threads(t)
        Cw = C.copy()
        oracle.gemm_work("N", "T", m, n, k, 1.5, A, lda, B, ldb, -0.5, Cw, ldc)
        outs.append(Cw)
    oracle.set_num_threads(nt)
    assert np.array_equal(outs[0], outs[1])


# --------------------------------------------------------------------------
# 7. complex GEMM on split planes
# --------------------------------------------------------------------------
def zoperands(rng, ta, tb, m, n, k, kind="int", pad=(1, 2, 3)):
    ra, ca = stored(ta, m, k)
    rb, cb = stored(tb, k, n)
    lda, ldb, ldc = ra + pad[0], rb + pad[1], m + pad[2]
    if kind == "int":
        gen = lambda r, c, ld: si.integers(rng, r, c, ld, R=100)
    else:
        gen = lambda r, c, ld: si.uniform(rng, r, c, ld)
    planes = [gen(ra, ca, lda), gen(ra, ca, lda), gen(rb, cb, ldb), gen(rb, cb, ldb),
              gen(m, n, ldc), gen(m, n, ldc)]
    return planes, lda, ldb, ldc


def zop(Xr, Xi, trans, rows_op, cols_op):
    r, _ = stored(trans, rows_op, cols_op)
    Z = si.view(Xr, r) + 1j * si.view(Xi, r)
    if trans in "Nn":
        return Z
    return Z.T.conj() if trans in "Cc" else Z.T


@pytest.mark.parametrize("ta,tb", list(itertools.product("NTC", "NTC")))
def test_zgemm_gaussian_integers_bit_exact(ta, tb):
    rng = si.rng_for(90, 14)
    m, n, k = 17, 13, 29
    (Ar, Ai, Br, Bi, Cr, Ci), lda, ldb, ldc = zoperands(rng, ta, tb, m, n, k)
    for alpha, beta in [((1, 0), (0, 0)), ((2, -1), (1, 3)), ((0, 0), (0, 1)), ((0, 1), (1, 0))]:
        # exact product in integer arithmetic (python ints via object arrays)
        ZA = zop(Ar, Ai, ta, m, k)
        ZB = zop(Br, Bi, tb, k, n)
        ar, ai = ZA.real.astype(np.int64), ZA.imag.astype(np.int64)
        br, bi = ZB.real.astype(np.int64), ZB.imag.astype(np.int64)
        pr, pi = ar @ br - ai @ bi, ar @ bi + ai @ br
        c0, c1 = si.view(Cr, m).astype(np.int64), si.view(Ci, m).astype(np.int64)
        wr = alpha[0] * pr - alpha[1] * pi + beta[0] * c0 - beta[1] * c1
        wi = alpha[0] * pi + alpha[1] * pr + beta[0] * c1 + beta[1] * c0
        info, Rr, Ri, Gr, Gi = oracle.zgemm_split_ext(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb,
                                                      beta, Cr, Ci, ldc)
        assert info == 0
        assert np.array_equal(Rr.T, wr.astype(np.longdouble)) and np.array_equal(Ri.T, wi.astype(np.longdouble))
        Wr, Wi = Cr.copy(), Ci.copy()
        assert oracle.zgemm_split_work(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Wr, Wi, ldc) == 0
        assert np.array_equal(si.view(Wr, m), wr.astype(np.float64))
        assert np.array_equal(si.view(Wi, m), wi.astype(np.float64))
        assert np.all(np.isnan(Wr[:, m:])) and np.all(np.isnan(Wi[:, m:]))


def test_zgemm_against_numpy_complex_and_real_special_case():
    rng = si.rng_for(90, 15)
    m, n, k = 24, 31, 57
    (Ar, Ai, Br, Bi, Cr, Ci), lda, ldb, ldc = zoperands(rng, "N", "C", m, n, k, kind="uniform")
    alpha, beta = (0.75, -1.25), (0.5, 2.0)
    info, Rr, Ri, Gr, Gi = oracle.zgemm_split_ext("N", "C", m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb,
                                                  beta, Cr, Ci, ldc)
    assert info == 0
    Z = complex(*alpha) * (zop(Ar, Ai, "N", m, k) @ zop(Br, Bi, "C", k, n)) \
        + complex(*beta) * (si.view(Cr, m) + 1j * si.view(Ci, m))
    assert np.all(np.abs(Z.real - Rr.T.astype(np.float64)) <= 8 * k * oracle.U64 * Gr.T.astype(np.float64))
    assert np.all(np.abs(Z.imag - Ri.T.astype(np.float64)) <= 8 * k * oracle.U64 * Gi.T.astype(np.float64))
    # zero imaginary planes reduce to the real GEMM reference exactly
    Z0 = np.zeros_like(Ai); Zb = np.zeros_like(Bi); Zc = np.zeros_like(Ci)
    info, Rr, Ri, Gr, Gi = oracle.zgemm_split_ext("N", "T", m, n, k, (1.5, 0.0), Ar, Z0, lda, Br, Zb, ldb,
                                                  (-0.5, 0.0), Cr, Zc, ldc)
    _, Cref, G = oracle.gemm_ext("N", "T", m, n, k, 1.5, Ar, lda, Br, ldb, -0.5, Cr, ldc)
    assert np.array_equal(Rr, Cref) and np.array_equal(Gr, G) and not Ri.any()


def test_zgemm_samples_match_full_reference():
    rng = si.rng_for(90, 16)
    m, n, k = 21, 19, 33
    for ta, tb in [("N", "N"), ("C", "T"), ("T", "C")]:
        (Ar, Ai, Br, Bi, Cr, Ci), lda, ldb, ldc = zoperands(rng, ta, tb, m, n, k, kind="uniform")
        al, be = (1.5, -0.25), (0.5, 1.0)
        _, Rr, Ri, Gr, Gi = oracle.zgemm_split_ext(ta, tb, m, n, k, al, Ar, Ai, lda, Br, Bi, ldb, be, Cr, Ci, ldc)
        I, J = si.sample_indices(rng, m, n, 3, 3, 40)
        info, rr, ri, gr, gi = oracle.zgemm_split_samples(ta, tb, m, n, k, al, Ar, Ai, lda, Br, Bi, ldb, be,
                                                          Cr, Ci, ldc, I, J)
        assert info == 0
        assert np.array_equal(rr, Rr[J, I]) and np.array_equal(ri, Ri[J, I])
        assert np.array_equal(gr, Gr[J, I]) and np.array_equal(gi, Gi[J, I])


def test_zgemm_scalar_paths_and_errors():
    m, n, k = 5, 4, 3
    nan = np.full((8, 8), np.nan)
    one = np.ones((8, 8))
    Cr, Ci = nan.copy(), nan.copy()
    # beta == 0 overwrites NaN
    assert oracle.zgemm_split_work("N", "N", m, n, k, (1, 0), one, one, 8, one, one, 8, (0, 0), Cr, Ci, 8) == 0
    assert np.array_equal(Cr[:n, :m], np.zeros((n, m))) and np.array_equal(Ci[:n, :m], np.full((n, m), 2.0 * k))
    # alpha == 0 does not read A, B
    Cr, Ci = one.copy(), 2 * one.copy()
    assert oracle.zgemm_split_work("N", "N", m, n, k, (0, 0), nan, nan, 8, nan, nan, 8, (0, 1), Cr, Ci, 8) == 0
    assert np.array_equal(Cr[:n, :m], np.full((n, m), -2.0)) and np.array_equal(Ci[:n, :m], np.ones((n, m)))
    z = oracle.zgemm_split_work
    assert z("X", "N", m, n, k, (1, 0), one, one, 8, one, one, 8, (0, 0), Cr, Ci, 8) == -1
    assert z("N", "N", m, n, k, (1, 0), one, None, 8, one, one, 8, (0, 0), Cr, Ci, 8) == -8
    assert z("N", "N", m, n, k, (1, 0), one, one, 4, one, one, 8, (0, 0), Cr, Ci, 8) == -9
    assert z("N", "N", m, n, k, (1, 0), one, one, 8, one, one, 2, (0, 0), Cr, Ci, 8) == -12
    assert z("N", "N", m, n, k, (1, 0), one, one, 8, one, one, 8, (0, 0), Cr, None, 8) == -15
    assert z("N", "N", m, n, k, (1, 0), one, one, 8, one, one, 8, (0, 0), Cr, Ci, 4) == -16
