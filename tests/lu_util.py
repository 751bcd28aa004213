"""Helpers shared by the LU pins (CPU) and the LU parity tests (GPU): matrices whose factorisation is
known exactly, and the validity statement of a factorisation with partial pivoting."""
import numpy as np

import oracle


def planted_lu(rng, m, n, dtype=np.float64, ld=None):
    """A matrix whose LU factorisation with partial pivoting is known exactly and is computed without any
    rounding, whatever the order of the operations: L has entries that are multiples of 1/4 in [-1/2, 1/2]
    below a unit diagonal, U has small integers above a diagonal of signed powers of two (4, 8 or 16), the
    product L U is taken exactly and its rows are shuffled.  In every column the pivot (|u_jj| >= 4) is more
    than twice any other candidate (|l_ij u_jj| <= |u_jj| / 2), so there are no ties.  Returns (A in the
    (col, ld) layout with NaN padding, L (m x k), U (k x n), perm) with (A[perm, :] as a matrix) == L U."""
    k = min(m, n)
    L = np.tril(rng.integers(-2, 3, size=(m, k)).astype(np.float64) / 4.0, -1)
    L[np.arange(k), np.arange(k)] = 1.0
    U = np.triu(rng.integers(-3, 4, size=(k, n)).astype(np.float64), 1)
    U[np.arange(k), np.arange(k)] = (2.0 ** rng.integers(2, 5, size=k)) * rng.choice([-1.0, 1.0], size=k)
    PA = L @ U                                         # exact: dyadic numbers of a few bits
    assert np.all(PA * 4 == np.round(PA * 4)) and np.abs(PA).max() < 2 ** 20
    perm = rng.permutation(m)                          # row i of P A is row perm[i] of A
    Amat = np.empty_like(PA)
    Amat[perm, :] = PA
    ld = m if ld is None else ld
    A = np.full((n, ld), np.nan, dtype=dtype)
    A[:, :m] = Amat.T.astype(dtype)
    return A, L, U, perm


def perm_of(ipiv, m):
    """Row i of P A is row src[i] of A after the interchanges ipiv[0], ipiv[1], ... (1-based) in that order."""
    src = np.arange(m)
    for j, p in enumerate(np.asarray(ipiv, dtype=np.int64) - 1):
        src[j], src[p] = src[p], src[j]
    return src


def unpack(F, m, n):
    """(L, U) as dense matrices from the packed factor in the (col, ld) layout."""
    k = min(m, n)
    M = F[:, :m].T.astype(np.float64)
    L = np.tril(M[:, :k], -1)
    L[np.arange(k), np.arange(k)] = 1.0
    return L, np.triu(M[:k, :])


def check_valid(m, n, A0, lda, F, ldf, ipiv, u, factor=4.0, I=None, J=None):
    """The statement every correct factorisation with partial pivoting satisfies, whatever the order of its
    sums and however ties were broken: ipiv is a legal sequence of interchanges, no multiplier exceeds one in
    magnitude, and |P A - L U| <= factor * min(m, n) * u * |L||U| element by element (on every element, or on
    the entries (I, J)).  Returns the largest err / bound."""
    k = min(m, n)
    ipiv = np.asarray(ipiv)
    assert ipiv.shape == (k,)
    assert np.all(ipiv >= np.arange(1, k + 1)) and np.all(ipiv <= m), "illegal interchange"
    M = F[:, :m]                                       # M[c, r] = F(r, c)
    c, r = np.meshgrid(np.arange(n), np.arange(m), indexing="ij")
    below = (r > c) & (c < k)
    assert np.all(np.abs(M[below]) <= 1.0), "a multiplier exceeds one: not a partial-pivoting factor"
    info, R, G = oracle.getrf_resid(m, n, A0, lda, F, ldf, ipiv, I, J)
    assert info == 0, info
    bound = factor * max(k, 1) * u * G
    bad = np.abs(R) > bound
    ratio = float(np.max(np.abs(R) / np.maximum(bound, np.finfo(np.float64).tiny))) if R.size else 0.0
    assert not bad.any(), f"{int(bad.sum())} entries outside the residual bound (max ratio {ratio})"
    return ratio
