"""CPU oracle for GEMM (ctypes front end of ``ref_gemm.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the GPU library never does, and
this package imports nothing from it.

The arithmetic lives in ``ref_gemm.c`` (plain C, triple loops; see its header
for the definition it writes out, paper Sec. 2.1).  This module only compiles
it with gcc, marshals numpy arrays, and offers the element-wise bound check
``|C - C_ref| <= 4 k u G``.

All matrices are column-major: a numpy array ``X`` of shape ``(cols, ld)`` in C
order holds element (i, j) at ``X[j, i]`` which is flat index ``i + j*ld``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ref_gemm.c")
_LIB = os.path.join(_HERE, "libref_gemm.so")

U64 = 2.0 ** -53  # unit roundoff, fp64
U32 = 2.0 ** -24  # unit roundoff, fp32


def build(force: bool = False) -> str:
    """Compile ref_gemm.c into libref_gemm.so (gcc, OpenMP, no FMA contraction)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _declare(_lib)
    return _lib


_i64 = ctypes.c_longlong
_p = ctypes.c_void_p


def _declare(L):
    for name, sc in (("ref_dgemm_work", ctypes.c_double), ("ref_sgemm_work", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, _i64, sc, _p, _i64, _p, _i64,
                      sc, _p, _i64]
    for name, sc in (("ref_dgemm_ext", ctypes.c_double), ("ref_sgemm_ext", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, _i64, sc, _p, _i64, _p, _i64,
                      sc, _p, _i64, _p, _p]
    for name, sc in (("ref_dgemm_samples", ctypes.c_double), ("ref_sgemm_samples", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, _i64, sc, _p, _i64, _p, _i64,
                      sc, _p, _i64, _i64, _p, _p, _p, _p]
    for name, sc in (("ref_dsyrk_work", ctypes.c_double), ("ref_ssyrk_work", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, sc, _p, _i64, sc, _p, _i64]
    for name, sc in (("ref_dsyrk_ext", ctypes.c_double), ("ref_ssyrk_ext", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, sc, _p, _i64, sc, _p, _i64, _p, _p]
    for name, sc in (("ref_dtrsm_work", ctypes.c_double), ("ref_strsm_work", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char] * 4 + [_i64, _i64, sc, _p, _i64, _p, _i64]
    for name, sc in (("ref_dtrsm_resid", ctypes.c_double), ("ref_strsm_resid", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char] * 4 + [_i64, _i64, sc, _p, _i64, _p, _i64, _p, _i64, _p, _p]
    for name, sc in (("ref_dtrsm_resid_samples", ctypes.c_double), ("ref_strsm_resid_samples", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char] * 4 + [_i64, _i64, sc, _p, _i64, _p, _i64, _p, _i64, _i64, _p, _p, _p, _p]
    for name, sc in (("ref_dtrmm_ext", ctypes.c_double), ("ref_strmm_ext", ctypes.c_float),
                     ("ref_dtrmm_wp", ctypes.c_double), ("ref_strmm_wp", ctypes.c_float)):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char] * 4 + [_i64, _i64, sc, _p, _i64, _p, _i64, _p, _p]
    for name in ("ref_dpotrf", "ref_spotrf"):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char, _i64, _p, _i64]
    for name in ("ref_dpotrf_resid", "ref_spotrf_resid"):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [ctypes.c_char, _i64, _p, _i64, _p, _i64, _i64, _p, _p, _p, _p]
    for name in ("ref_dgetrf", "ref_sgetrf"):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [_i64, _i64, _p, _i64, _p]
    for name in ("ref_dgetrf_resid", "ref_sgetrf_resid"):
        f = getattr(L, name)
        f.restype = ctypes.c_int
        f.argtypes = [_i64, _i64, _p, _i64, _p, _i64, _p, _i64, _p, _p, _p, _p]
    for pre, sc in (("d", ctypes.c_double), ("s", ctypes.c_float)):
        for suf in ("ext", "wp"):
            f = getattr(L, f"ref_{pre}syr2k_{suf}")
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, sc, _p, _i64, _p, _i64, sc, _p, _i64, _p, _p]
            f = getattr(L, f"ref_{pre}symm_{suf}")
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, sc, _p, _i64, _p, _i64, sc, _p, _i64, _p, _p]
    L.ref_zgemm_split_ext.restype = ctypes.c_int
    L.ref_zgemm_split_ext.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, _i64, _p,
                                      _p, _p, _i64, _p, _p, _i64, _p, _p, _p, _i64,
                                      _p, _p, _p, _p]
    L.ref_zgemm_split_samples.restype = ctypes.c_int
    L.ref_zgemm_split_samples.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, _i64, _p,
                                          _p, _p, _i64, _p, _p, _i64, _p, _p, _p, _i64,
                                          _i64, _p, _p, _p, _p, _p, _p]
    L.ref_zgemm_split_work.restype = ctypes.c_int
    L.ref_zgemm_split_work.argtypes = [ctypes.c_char, ctypes.c_char, _i64, _i64, _i64, _p,
                                       _p, _p, _i64, _p, _p, _i64, _p, _p, _p, _i64]
    L.ref_num_threads.restype = ctypes.c_int
    L.ref_set_num_threads.argtypes = [ctypes.c_int]


def num_threads() -> int:
    return int(lib().ref_num_threads())


def set_num_threads(t: int) -> None:
    lib().ref_set_num_threads(int(t))


def _ptr(a):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def _ch(t: str):
    return ctypes.c_char(t.encode("ascii"))


def _names(dtype):
    dtype = np.dtype(dtype)
    if dtype == np.float64:
        return "d", np.longdouble
    if dtype == np.float32:
        return "s", np.float64
    raise TypeError(f"unsupported dtype {dtype}")


def gemm_work(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc) -> int:
    """In-place working-precision GEMM on C (numpy, column-major flat storage)."""
    pre, _ = _names(C.dtype if C is not None else (A.dtype if A is not None else np.float64))
    f = getattr(lib(), f"ref_{pre}gemm_work")
    return int(f(_ch(ta), _ch(tb), m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc))


def gemm_ext(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc):
    """Extended-precision reference.  Returns (info, Cref, G); Cref/G have shape
    (n, m) in C order (= m x n column-major, ld = m) in the wide dtype."""
    pre, wide = _names(C.dtype)
    Cref = np.zeros((max(n, 0), max(m, 0)), dtype=wide)
    G = np.zeros_like(Cref)
    f = getattr(lib(), f"ref_{pre}gemm_ext")
    info = int(f(_ch(ta), _ch(tb), m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                 _ptr(Cref), _ptr(G)))
    return info, Cref, G


def gemm_samples(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, I, J):
    """Extended-precision reference for entries (I[s], J[s]).  Returns (info, cref, g)."""
    pre, wide = _names(C.dtype)
    I = np.ascontiguousarray(I, dtype=np.int64)
    J = np.ascontiguousarray(J, dtype=np.int64)
    ns = I.size
    cref = np.zeros(ns, dtype=wide)
    g = np.zeros(ns, dtype=wide)
    f = getattr(lib(), f"ref_{pre}gemm_samples")
    info = int(f(_ch(ta), _ch(tb), m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                 ns, _ptr(I), _ptr(J), _ptr(cref), _ptr(g)))
    return info, cref, g


def syrk_work(uplo, trans, n, k, alpha, A, lda, beta, C, ldc) -> int:
    """In-place working-precision symmetric rank-k update of one triangle of C."""
    pre, _ = _names(C.dtype if C is not None else np.float64)
    f = getattr(lib(), f"ref_{pre}syrk_work")
    return int(f(_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, beta, _ptr(C), ldc))


def syrk_ext(uplo, trans, n, k, alpha, A, lda, beta, C, ldc):
    """Extended-precision reference; returns (info, Cref, G), shape (n, n), zero outside the triangle."""
    pre, wide = _names(C.dtype)
    Cref = np.zeros((max(n, 0), max(n, 0)), dtype=wide)
    G = np.zeros_like(Cref)
    f = getattr(lib(), f"ref_{pre}syrk_ext")
    info = int(f(_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, beta, _ptr(C), ldc, _ptr(Cref), _ptr(G)))
    return info, Cref, G


def triangle_mask(uplo, n):
    """Boolean (n, n) mask in the (col, row) array layout: True where C(i, j) belongs to the triangle."""
    j, i = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    return (i >= j) if uplo in "Ll" else (i <= j)


def trsm_work(side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb) -> int:
    """In-place working-precision triangular solve: B <- X with op(T) X = alpha B (L) or X op(T) = alpha B (R)."""
    pre, _ = _names(B.dtype if B is not None else np.float64)
    f = getattr(lib(), f"ref_{pre}trsm_work")
    return int(f(_ch(side), _ch(uplo), _ch(trans), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B), ldb))


def trsm_resid(side, uplo, trans, diag, m, n, alpha, A, lda, B0, ldb, X, ldx):
    """Extended-precision residual of a candidate X; returns (info, R, G), each of shape (n, m)."""
    pre, wide = _names(B0.dtype)
    R = np.zeros((max(n, 0), max(m, 0)), dtype=wide)
    G = np.zeros_like(R)
    f = getattr(lib(), f"ref_{pre}trsm_resid")
    info = int(f(_ch(side), _ch(uplo), _ch(trans), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B0), ldb,
                 _ptr(X), ldx, _ptr(R), _ptr(G)))
    return info, R, G


def trsm_resid_samples(side, uplo, trans, diag, m, n, alpha, A, lda, B0, ldb, X, ldx, I, J):
    """The residual at the entries (I[s], J[s]) only; returns (info, R, G) as 1-d arrays."""
    pre, wide = _names(B0.dtype)
    I = np.ascontiguousarray(I, dtype=np.int64)
    J = np.ascontiguousarray(J, dtype=np.int64)
    R = np.zeros(I.size, dtype=wide)
    G = np.zeros(I.size, dtype=wide)
    f = getattr(lib(), f"ref_{pre}trsm_resid_samples")
    info = int(f(_ch(side), _ch(uplo), _ch(trans), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B0), ldb,
                 _ptr(X), ldx, I.size, _ptr(I), _ptr(J), _ptr(R), _ptr(G)))
    return info, R, G


def trmm_ext(side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb):
    """alpha op(T) B (side L) or alpha B op(T) (side R) in extended precision; returns (info, Out, G), shape (n, m)."""
    pre, wide = _names(B.dtype)
    Out = np.zeros((max(n, 0), max(m, 0)), dtype=wide)
    G = np.zeros_like(Out)
    f = getattr(lib(), f"ref_{pre}trmm_ext")
    info = int(f(_ch(side), _ch(uplo), _ch(trans), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B), ldb,
                 _ptr(Out), _ptr(G)))
    return info, Out, G


def trmm_work(side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb) -> int:
    """Working-precision triangular product, B overwritten (through a dense temporary)."""
    if B is None:
        f = lib().ref_dtrmm_wp
        return int(f(_ch(side), _ch(uplo), _ch(trans), _ch(diag), m, n, alpha, _ptr(A), lda, None, ldb, None, None))
    pre, _ = _names(B.dtype)
    Out = np.zeros((max(n, 0), max(m, 0)), dtype=B.dtype)
    G = np.zeros_like(Out)
    f = getattr(lib(), f"ref_{pre}trmm_wp")
    info = int(f(_ch(side), _ch(uplo), _ch(trans), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B), ldb,
                 _ptr(Out), _ptr(G)))
    if info == 0 and m > 0 and n > 0:
        B[:, :m] = Out
    return info


def potrf(uplo, n, A, lda) -> int:
    """In-place working-precision Cholesky factorisation of the `uplo` triangle; returns LAPACK's info."""
    pre, _ = _names(A.dtype if A is not None else np.float64)
    return int(getattr(lib(), f"ref_{pre}potrf")(_ch(uplo), n, _ptr(A), lda))


def potrf_resid(uplo, n, A0, lda, F, ldf, I=None, J=None):
    """Extended-precision residual A0 - L L^T and magnitude |L||L|^T of a candidate factor on the
    triangle: dense (n, n) arrays in the (col, row) layout, or 1-d arrays at the entries (I, J)."""
    pre, wide = _names(A0.dtype)
    f = getattr(lib(), f"ref_{pre}potrf_resid")
    if I is None:
        R = np.zeros((max(n, 0), max(n, 0)), dtype=wide)
        G = np.zeros_like(R)
        info = int(f(_ch(uplo), n, _ptr(A0), lda, _ptr(F), ldf, -1, None, None, _ptr(R), _ptr(G)))
        return info, R, G
    I = np.ascontiguousarray(I, dtype=np.int64)
    J = np.ascontiguousarray(J, dtype=np.int64)
    R = np.zeros(I.size, dtype=wide)
    G = np.zeros(I.size, dtype=wide)
    info = int(f(_ch(uplo), n, _ptr(A0), lda, _ptr(F), ldf, I.size, _ptr(I), _ptr(J), _ptr(R), _ptr(G)))
    return info, R, G


def getrf(m, n, A, lda):
    """In-place working-precision LU with partial pivoting (first largest entry of the column); returns
    (info, ipiv) with ipiv 1-based int32 of length min(m, n), LAPACK's conventions."""
    pre, _ = _names(A.dtype if A is not None else np.float64)
    ipiv = np.zeros(max(min(m, n), 0), dtype=np.int32)
    info = int(getattr(lib(), f"ref_{pre}getrf")(m, n, _ptr(A), lda, _ptr(ipiv) if ipiv.size else None))
    return info, ipiv


def getrf_resid(m, n, A0, lda, F, ldf, ipiv, I=None, J=None):
    """Extended-precision residual P A0 - L U and magnitude |L||U| of a candidate factorisation:
    dense (n, m) arrays in the (col, row) layout, or 1-d arrays at the entries (I, J)."""
    pre, wide = _names(A0.dtype)
    f = getattr(lib(), f"ref_{pre}getrf_resid")
    ipiv = np.ascontiguousarray(ipiv, dtype=np.int32)
    if I is None:
        R = np.zeros((max(n, 0), max(m, 0)), dtype=wide)
        G = np.zeros_like(R)
        info = int(f(m, n, _ptr(A0), lda, _ptr(F), ldf, _ptr(ipiv), -1, None, None, _ptr(R), _ptr(G)))
        return info, R, G
    I = np.ascontiguousarray(I, dtype=np.int64)
    J = np.ascontiguousarray(J, dtype=np.int64)
    R = np.zeros(I.size, dtype=wide)
    G = np.zeros(I.size, dtype=wide)
    info = int(f(m, n, _ptr(A0), lda, _ptr(F), ldf, _ptr(ipiv), I.size, _ptr(I), _ptr(J), _ptr(R), _ptr(G)))
    return info, R, G


def _dense_pair(fname, dtype, rows, cols, args):
    Out = np.zeros((max(cols, 0), max(rows, 0)), dtype=dtype)
    G = np.zeros_like(Out)
    info = int(getattr(lib(), fname)(*args, _ptr(Out), _ptr(G)))
    return info, Out, G


def syr2k_ext(uplo, trans, n, k, alpha, A, lda, B, ldb, beta, C, ldc):
    """Extended-precision rank-2k update of one triangle; (info, Cref, G), shape (n, n), zero outside the triangle."""
    pre, wide = _names(C.dtype)
    return _dense_pair(f"ref_{pre}syr2k_ext", wide, n, n,
                       (_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc))


def syr2k_work(uplo, trans, n, k, alpha, A, lda, B, ldb, beta, C, ldc) -> int:
    """Working-precision rank-2k update; the triangle of C is overwritten."""
    if C is None:
        return int(lib().ref_dsyr2k_wp(_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta, None, ldc,
                                       None, None))
    pre, _ = _names(C.dtype)
    info, Out, _g = _dense_pair(f"ref_{pre}syr2k_wp", C.dtype, n, n,
                                (_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc))
    if info == 0 and n > 0:
        mask = triangle_mask(uplo, n)
        C[:, :n][mask] = Out[mask]
    return info


def symm_ext(side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc):
    """Extended-precision symmetric product; (info, Cref, G), shape (n, m)."""
    pre, wide = _names(C.dtype)
    return _dense_pair(f"ref_{pre}symm_ext", wide, m, n,
                       (_ch(side), _ch(uplo), m, n, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc))


def symm_work(side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc) -> int:
    """Working-precision symmetric product; C is overwritten."""
    if C is None:
        return int(lib().ref_dsymm_wp(_ch(side), _ch(uplo), m, n, alpha, _ptr(A), lda, _ptr(B), ldb, beta, None, ldc,
                                      None, None))
    pre, _ = _names(C.dtype)
    info, Out, _g = _dense_pair(f"ref_{pre}symm_wp", C.dtype, m, n,
                                (_ch(side), _ch(uplo), m, n, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc))
    if info == 0 and m > 0 and n > 0:
        C[:, :m] = Out
    return info


def zgemm_split_ext(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc):
    """Complex reference on split planes.  Returns (info, Rr, Ri, Gr, Gi), long double, (n, m)."""
    al = np.array(alpha, dtype=np.float64)
    be = np.array(beta, dtype=np.float64)
    shp = (max(n, 0), max(m, 0))
    Rr, Ri, Gr, Gi = (np.zeros(shp, dtype=np.longdouble) for _ in range(4))
    info = int(lib().ref_zgemm_split_ext(_ch(ta), _ch(tb), m, n, k, _ptr(al), _ptr(Ar), _ptr(Ai), lda,
                                         _ptr(Br), _ptr(Bi), ldb, _ptr(be), _ptr(Cr), _ptr(Ci), ldc,
                                         _ptr(Rr), _ptr(Ri), _ptr(Gr), _ptr(Gi)))
    return info, Rr, Ri, Gr, Gi


def zgemm_split_samples(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc, I, J):
    """Entries (I[s], J[s]) of the complex reference.  Returns (info, rr, ri, gr, gi)."""
    al = np.array(alpha, dtype=np.float64)
    be = np.array(beta, dtype=np.float64)
    I = np.ascontiguousarray(I, dtype=np.int64)
    J = np.ascontiguousarray(J, dtype=np.int64)
    rr, ri, gr, gi = (np.zeros(I.size, dtype=np.longdouble) for _ in range(4))
    info = int(lib().ref_zgemm_split_samples(_ch(ta), _ch(tb), m, n, k, _ptr(al), _ptr(Ar), _ptr(Ai), lda,
                                             _ptr(Br), _ptr(Bi), ldb, _ptr(be), _ptr(Cr), _ptr(Ci), ldc,
                                             I.size, _ptr(I), _ptr(J), _ptr(rr), _ptr(ri), _ptr(gr), _ptr(gi)))
    return info, rr, ri, gr, gi


def zgemm_split_work(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc) -> int:
    al = np.array(alpha, dtype=np.float64)
    be = np.array(beta, dtype=np.float64)
    return int(lib().ref_zgemm_split_work(_ch(ta), _ch(tb), m, n, k, _ptr(al), _ptr(Ar), _ptr(Ai), lda,
                                          _ptr(Br), _ptr(Bi), ldb, _ptr(be), _ptr(Cr), _ptr(Ci), ldc))


def bound_violations(C_test, C_ref, G, k, u, factor=4.0):
    """Element-wise check |C_test - C_ref| <= factor * k * u * G, evaluated in the
    wide dtype of C_ref.  Returns (number of violations, max of err / bound with
    0/0 counted as 0).  ``k`` below 1 is treated as 1 (the alpha/beta roundings
    remain when the product term is absent)."""
    wide = C_ref.dtype
    err = np.abs(C_test.astype(wide) - C_ref)
    bnd = wide.type(factor * max(int(k), 1) * u) * G
    viol = err > bnd
    # NaN in the tested values must count as a violation.
    viol |= ~np.isfinite(C_test)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(bnd > 0, err / bnd, np.where(err > 0, np.inf, 0.0))
    return int(viol.sum()), float(ratio.max()) if ratio.size else 0.0
