"""Seeded synthetic GEMM inputs shared by the tests, the smoke check and bench.py.

This module holds no GEMM arithmetic: it only draws numbers and lays them out
column-major.  Both the CPU oracle side and the GPU side of a parity test take
their operands from here, so they see the same bits.

Layout: a column-major ``rows x cols`` matrix with leading dimension ``ld`` is
a numpy array of shape ``(cols, ld)`` in C order; element (i, j) is ``X[j, i]``
(flat index ``i + j*ld``).  Rows ``rows..ld-1`` of every column are padding and
are filled with a sentinel (NaN by default) so that any read of the padding
shows up in the result.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 16110835  # seed = BASE_SEED + 1000*config + index


def seed_for(config: int, index: int = 0) -> int:
    return BASE_SEED + 1000 * int(config) + int(index)


def padded_ld(dim: int, multiple: int = 8) -> int:
    """Smallest multiple of ``multiple`` strictly above ``dim`` (8192 -> 8200)."""
    return multiple * ((dim + multiple) // multiple)


def _alloc(rows, cols, ld, dtype, sentinel):
    ld = max(int(ld), 1)
    X = np.empty((cols, ld), dtype=dtype)
    if ld > rows:
        X[:, rows:] = sentinel
    return X


def uniform(rng, rows, cols, ld=None, dtype=np.float64, lo=-1.0, hi=1.0, sentinel=np.nan):
    ld = rows if ld is None else ld
    X = _alloc(rows, cols, ld, dtype, sentinel)
    X[:, :rows] = rng.uniform(lo, hi, size=(cols, rows)).astype(dtype)
    return X


def normal(rng, rows, cols, ld=None, dtype=np.float64, sentinel=np.nan):
    ld = rows if ld is None else ld
    X = _alloc(rows, cols, ld, dtype, sentinel)
    X[:, :rows] = rng.standard_normal(size=(cols, rows)).astype(dtype)
    return X


def integers(rng, rows, cols, ld=None, dtype=np.float64, R=8, sentinel=np.nan):
    """Integer-valued entries in [-R, R] stored in a floating dtype."""
    ld = rows if ld is None else ld
    X = _alloc(rows, cols, ld, dtype, sentinel)
    X[:, :rows] = rng.integers(-R, R + 1, size=(cols, rows)).astype(dtype)
    return X


def constant(rows, cols, ld=None, dtype=np.float64, value=1.0, sentinel=np.nan):
    ld = rows if ld is None else ld
    X = _alloc(rows, cols, ld, dtype, sentinel)
    X[:, :rows] = value
    return X


def identity(nrows, ld=None, dtype=np.float64, sentinel=np.nan):
    ld = nrows if ld is None else ld
    X = _alloc(nrows, nrows, ld, dtype, sentinel)
    X[:, :nrows] = np.eye(nrows, dtype=dtype)
    return X


def _mask_triangle(X, n, uplo, unit_diag, sentinel):
    """Overwrite everything the triangular routines must not read with the sentinel."""
    j, i = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    outside = (i < j) if uplo in "Ll" else (i > j)
    if unit_diag:
        outside |= (i == j)
    X[:, :n][outside] = sentinel
    return X


def triangular(rng, n, ld=None, dtype=np.float64, uplo="L", unit_diag=False, sentinel=np.nan):
    """Well-conditioned triangular factor of the kind a pivoted LU or a Cholesky
    factorisation leaves behind: off-diagonal entries uniform in [-1, 1] / n,
    diagonal uniform in [1, 2] (or implicit ones).  The other triangle, the
    diagonal of a unit-diagonal matrix and the padding hold the sentinel."""
    ld = n if ld is None else ld
    X = _alloc(n, n, ld, dtype, sentinel)
    X[:, :n] = (rng.uniform(-1.0, 1.0, size=(n, n)) / max(n, 1)).astype(dtype)
    d = rng.uniform(1.0, 2.0, size=n).astype(dtype)
    X[np.arange(n), np.arange(n)] = d
    return _mask_triangle(X, n, uplo, unit_diag, sentinel)


def int_triangular(rng, n, ld=None, dtype=np.float64, uplo="L", unit_diag=False, R=4, sentinel=np.nan):
    """Integer off-diagonal entries in [-R, R] and a diagonal of signed powers of
    two (1, 2 or 4): every quotient by a diagonal entry is exact."""
    ld = n if ld is None else ld
    X = _alloc(n, n, ld, dtype, sentinel)
    X[:, :n] = rng.integers(-R, R + 1, size=(n, n)).astype(dtype)
    d = (2.0 ** rng.integers(0, 3, size=n)) * rng.choice([-1.0, 1.0], size=n)
    X[np.arange(n), np.arange(n)] = d.astype(dtype)
    return _mask_triangle(X, n, uplo, unit_diag, sentinel)


def spd(rng, n, ld=None, dtype=np.float64, uplo="L", sentinel=np.nan):
    """Symmetric positive definite matrix given by one triangle: off-diagonal
    entries uniform in [-1, 1], diagonal n + uniform[0, 1] (strictly diagonally
    dominant, hence positive definite; condition number of order one).  The other
    triangle and the padding hold the sentinel."""
    ld = n if ld is None else ld
    X = _alloc(n, n, ld, dtype, sentinel)
    X[:, :n] = rng.uniform(-1.0, 1.0, size=(n, n)).astype(dtype)
    X[np.arange(n), np.arange(n)] = (n + rng.uniform(0.0, 1.0, size=n)).astype(dtype)
    return _mask_triangle(X, n, uplo, False, sentinel)


def rng_for(config: int, index: int = 0):
    return np.random.Generator(np.random.PCG64(seed_for(config, index)))


def operand_shape(trans: str, rows_op: int, cols_op: int):
    """Stored (rows, cols) of an operand whose op(X) is rows_op x cols_op."""
    return (rows_op, cols_op) if trans in "Nn" else (cols_op, rows_op)


def view(X, rows):
    """The logical rows x cols part as a (rows, cols) array (copy-free transpose view)."""
    return X[:, :rows].T


def sample_indices(rng, m, n, nrows=8, ncols=8, nrand=4096):
    """Entry list for sampled parity: a few full rows, a few full columns (always
    including the first and last of each) and random entries."""
    rows = np.unique(np.concatenate([[0, m - 1], rng.integers(0, m, size=max(nrows - 2, 0))]))
    cols = np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, size=max(ncols - 2, 0))]))
    I = [np.repeat(rows, n), np.tile(np.arange(m), cols.size), rng.integers(0, m, size=nrand)]
    J = [np.tile(np.arange(n), rows.size), np.repeat(cols, m), rng.integers(0, n, size=nrand)]
    return np.concatenate(I).astype(np.int64), np.concatenate(J).astype(np.int64)
