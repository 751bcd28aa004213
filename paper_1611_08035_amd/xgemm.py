"""ctypes binding of libxgemm.so -- same names as the C ABI (include/xgemm.h, xgemm_tuning.h, xgemm_probe.h).

Matrix arguments may be torch tensors on the GPU (their ``data_ptr()`` is
passed) or plain integer device addresses; ``None`` is a NULL pointer.  The
stream defaults to torch's current stream on the current device.  Nothing is
computed here.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "libxgemm.so")

EXPORTS = [
    "xgemm_dgemm", "xgemm_sgemm", "xgemm_dsyrk", "xgemm_ssyrk", "xgemm_zgemm_split", "xgemm_zgemm_worksize", "xgemm_version",
    "xgemm_last_kernel_name", "xgemm_force_variant", "xgemm_variant_name", "xgemm_mfma_peak_probe",
    "xgemm_mfma_layout_probe", "xgemm_hwid_probe", "xgemm_model_outer_product_rate",
    "xgemm_model_stalled_rate", "xgemm_model_n_updates", "xgemm_model_predict", "xgemm_tile_map",
    "xgemm_workspace_bytes", "xgemm_workspace_init", "xgemm_dgemm_ws", "xgemm_sgemm_ws", "xgemm_dsyrk_ws",
    "xgemm_ssyrk_ws", "xgemm_force_split", "xgemm_last_split", "xgemm_plan", "xgemm_dtrsm", "xgemm_strsm", "xgemm_dtrmm", "xgemm_strmm", "xgemm_dsyr2k", "xgemm_ssyr2k", "xgemm_dsymm",
    "xgemm_ssymm", "xgemm_zgemm", "xgemm_zgemm_workbytes", "xgemm_dpotrf", "xgemm_spotrf", "xgemm_latency_probe",
    "xgemm_force_potrf_panel", "xgemm_force_potrf_block", "xgemm_dgemm_static", "xgemm_tuning_reset", "xgemm_model_enumerate", "xgemm_model_efficiency", "xgemm_dgetrf", "xgemm_sgetrf", "xgemm_force_getrf_panel", "xgemm_dgetrf_ws", "xgemm_sgetrf_ws", "xgemm_getrf_workspace_bytes", "xgemm_force_getrf_spin_limit", "xgemm_force_getrf_poll_delay", "xgemm_force_getrf_shared", "xgemm_pack_elems", "xgemm_dpack_a", "xgemm_dpack_b", "xgemm_spack_a", "xgemm_spack_b", "xgemm_dgemm_packed", "xgemm_sgemm_packed", "xgemm_release_thread_resources",
]


class XgemmError(RuntimeError):
    pass


_lib = None
_i64, _p, _c = ctypes.c_int64, ctypes.c_void_p, ctypes.c_char


def library_path() -> str:
    return _LIBPATH


def lib():
    """Load libxgemm.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIBPATH):
        raise XgemmError(
            f"{_LIBPATH} is missing: build it with `python -m paper_1611_08035_amd.build` "
            "(there is no fallback path)")
    # torch brings its own HIP runtime; load it first so that this library
    # binds to the same runtime instance that owns the tensors' memory.
    try:
        import torch  # noqa: F401
    except Exception:
        pass
    L = ctypes.CDLL(_LIBPATH)
    for pre, sc in (("d", ctypes.c_double), ("s", ctypes.c_float)):
        f = getattr(L, f"xgemm_{pre}gemm")
        f.restype = ctypes.c_int
        f.argtypes = [_c, _c, _i64, _i64, _i64, sc, _p, _i64, _p, _i64, sc, _p, _i64, _p]
    L.xgemm_dgemm_static.restype = ctypes.c_int
    L.xgemm_dgemm_static.argtypes = L.xgemm_dgemm.argtypes
    for pre, sc in (("d", ctypes.c_double), ("s", ctypes.c_float)):
        f = getattr(L, f"xgemm_{pre}syrk")
        f.restype = ctypes.c_int
        f.argtypes = [_c, _c, _i64, _i64, sc, _p, _i64, sc, _p, _i64, _p]
    for pre, sc in (("d", ctypes.c_double), ("s", ctypes.c_float)):
        f = getattr(L, f"xgemm_{pre}gemm_ws")
        f.restype = ctypes.c_int
        f.argtypes = [_c, _c, _i64, _i64, _i64, sc, _p, _i64, _p, _i64, sc, _p, _i64, _p, ctypes.c_size_t, _p]
        f = getattr(L, f"xgemm_{pre}syrk_ws")
        f.restype = ctypes.c_int
        f.argtypes = [_c, _c, _i64, _i64, sc, _p, _i64, sc, _p, _i64, _p, ctypes.c_size_t, _p]
    for pre, sc in (("d", ctypes.c_double), ("s", ctypes.c_float)):
        for op in ("trsm", "trmm"):
            f = getattr(L, f"xgemm_{pre}{op}")
            f.restype = ctypes.c_int
            f.argtypes = [_c, _c, _c, _c, _i64, _i64, sc, _p, _i64, _p, _i64, _p]
    for pre in "ds":
        f = getattr(L, f"xgemm_{pre}potrf")
        f.restype = ctypes.c_int
        f.argtypes = [_c, _i64, _p, _i64, _p, _p]
    for pre in "ds":
        f = getattr(L, f"xgemm_{pre}getrf")
        f.restype = ctypes.c_int
        f.argtypes = [_i64, _i64, _p, _i64, _p, _p, _p]
    L.xgemm_pack_elems.restype = ctypes.c_size_t
    L.xgemm_pack_elems.argtypes = [_i64, _i64]
    for nm in ("xgemm_dpack_a", "xgemm_dpack_b", "xgemm_spack_a", "xgemm_spack_b"):
        f = getattr(L, nm)
        f.restype = ctypes.c_int
        f.argtypes = [_c, _i64, _i64, _p, _i64, _p, _p]
    for nm, ft in (("xgemm_dgemm_packed", ctypes.c_double), ("xgemm_sgemm_packed", ctypes.c_float)):
        f = getattr(L, nm)
        f.restype = ctypes.c_int
        f.argtypes = [_i64, _i64, _i64, ft, _p, _p, ft, _p, _i64, _p]
    for pre in ("d", "s"):
        f = getattr(L, f"xgemm_{pre}getrf_ws")
        f.restype = ctypes.c_int
        f.argtypes = [_i64, _i64, _p, _i64, _p, _p, _p, ctypes.c_size_t, _p]
    L.xgemm_getrf_workspace_bytes.restype = ctypes.c_size_t
    L.xgemm_getrf_workspace_bytes.argtypes = []
    L.xgemm_force_getrf_shared.restype = ctypes.c_int
    L.xgemm_force_getrf_shared.argtypes = [ctypes.c_int]
    L.xgemm_force_getrf_poll_delay.restype = ctypes.c_int
    L.xgemm_force_getrf_poll_delay.argtypes = [ctypes.c_int, ctypes.c_int]
    L.xgemm_force_getrf_spin_limit.restype = ctypes.c_int
    L.xgemm_force_getrf_spin_limit.argtypes = [ctypes.c_int]
    L.xgemm_force_getrf_panel.restype = ctypes.c_int
    L.xgemm_force_getrf_panel.argtypes = [ctypes.c_int64]
    for pre, sc in (("d", ctypes.c_double), ("s", ctypes.c_float)):
        for op in ("syr2k", "symm"):
            f = getattr(L, f"xgemm_{pre}{op}")
            f.restype = ctypes.c_int
            f.argtypes = [_c, _c, _i64, _i64, sc, _p, _i64, _p, _i64, sc, _p, _i64, _p]
    L.xgemm_zgemm.restype = ctypes.c_int
    L.xgemm_zgemm.argtypes = [_c, _c, _i64, _i64, _i64, _p, _p, _i64, _p, _i64, _p, _p, _i64, ctypes.c_int, _p,
                              ctypes.c_size_t, _p]
    L.xgemm_zgemm_workbytes.restype = ctypes.c_size_t
    L.xgemm_zgemm_workbytes.argtypes = [_i64, _i64, _i64, ctypes.c_int]
    L.xgemm_workspace_bytes.restype = ctypes.c_size_t
    L.xgemm_workspace_bytes.argtypes = []
    L.xgemm_workspace_init.restype = ctypes.c_int
    L.xgemm_workspace_init.argtypes = [_p, ctypes.c_size_t, _p]
    L.xgemm_force_split.restype = ctypes.c_int
    L.xgemm_force_split.argtypes = [ctypes.c_int]
    L.xgemm_last_split.restype = ctypes.c_int
    L.xgemm_plan.restype = ctypes.c_int
    L.xgemm_plan.argtypes = [_c, ctypes.c_int, _i64, _i64, _i64, ctypes.c_size_t, _p]
    L.xgemm_zgemm_split.restype = ctypes.c_int
    L.xgemm_zgemm_split.argtypes = [_c, _c, _i64, _i64, _i64, _p, _p, _p, _i64, _p, _p, _i64, _p, _p, _p, _i64,
                                    _p, _i64, _p]
    L.xgemm_zgemm_worksize.restype = ctypes.c_size_t
    L.xgemm_zgemm_worksize.argtypes = [_i64, _i64, _p, _p]
    L.xgemm_tile_map.restype = _i64
    L.xgemm_tile_map.argtypes = [ctypes.c_int, _i64, _i64, ctypes.c_int, ctypes.c_int, _p, _i64]
    L.xgemm_version.restype = ctypes.c_char_p
    L.xgemm_last_kernel_name.restype = ctypes.c_char_p
    L.xgemm_force_variant.restype = ctypes.c_int
    L.xgemm_force_variant.argtypes = [ctypes.c_int]
    L.xgemm_variant_name.restype = ctypes.c_char_p
    L.xgemm_variant_name.argtypes = [_c, ctypes.c_int]
    L.xgemm_mfma_peak_probe.restype = ctypes.c_int
    L.xgemm_mfma_peak_probe.argtypes = [_c, ctypes.c_int, ctypes.c_int, _p, _p]
    L.xgemm_mfma_layout_probe.restype = ctypes.c_int
    L.xgemm_mfma_layout_probe.argtypes = [_c, _p, _p]
    L.xgemm_hwid_probe.restype = ctypes.c_int
    L.xgemm_hwid_probe.argtypes = [ctypes.c_int, ctypes.c_int, _p, _p]
    L.xgemm_tuning_reset.restype = None
    L.xgemm_tuning_reset.argtypes = []
    L.xgemm_release_thread_resources.restype = ctypes.c_int
    L.xgemm_release_thread_resources.argtypes = []
    L.xgemm_force_potrf_block.restype = ctypes.c_int
    L.xgemm_force_potrf_block.argtypes = [ctypes.c_int]
    L.xgemm_force_potrf_panel.restype = ctypes.c_int
    L.xgemm_force_potrf_panel.argtypes = [ctypes.c_int64]
    L.xgemm_latency_probe.restype = ctypes.c_int
    L.xgemm_latency_probe.argtypes = [_p, _p, ctypes.c_int, _p]
    L.xgemm_model_outer_product_rate.restype = ctypes.c_double
    L.xgemm_model_outer_product_rate.argtypes = [ctypes.c_int, _p, _p]
    L.xgemm_model_stalled_rate.restype = ctypes.c_double
    L.xgemm_model_stalled_rate.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_double]
    L.xgemm_model_n_updates.restype = ctypes.c_int
    L.xgemm_model_n_updates.argtypes = [ctypes.c_int] * 6
    L.xgemm_model_efficiency.restype = ctypes.c_int
    L.xgemm_model_efficiency.argtypes = [_c, ctypes.c_int, _p]
    L.xgemm_model_enumerate.restype = ctypes.c_int
    L.xgemm_model_enumerate.argtypes = [_c, ctypes.c_int, _p]
    L.xgemm_model_predict.restype = ctypes.c_int
    L.xgemm_model_predict.argtypes = [_c, ctypes.c_int, _c, _c, _p]
    _lib = L
    return L


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()   # torch tensor


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ch(t):
    return _c(t.encode("ascii") if isinstance(t, str) else t)


def xgemm_dgemm(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream=None) -> int:
    return int(lib().xgemm_dgemm(_ch(transa), _ch(transb), m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                 _ptr(C), ldc, _stream(stream)))


def xgemm_sgemm(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream=None) -> int:
    return int(lib().xgemm_sgemm(_ch(transa), _ch(transb), m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                 _ptr(C), ldc, _stream(stream)))


def xgemm_dsyrk(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, stream=None) -> int:
    return int(lib().xgemm_dsyrk(_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, beta, _ptr(C), ldc,
                                 _stream(stream)))


def xgemm_ssyrk(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, stream=None) -> int:
    return int(lib().xgemm_ssyrk(_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, beta, _ptr(C), ldc,
                                 _stream(stream)))


def xgemm_dtrsm(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream=None) -> int:
    return int(lib().xgemm_dtrsm(_ch(side), _ch(uplo), _ch(transa), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B), ldb,
                                 _stream(stream)))


def xgemm_strsm(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream=None) -> int:
    return int(lib().xgemm_strsm(_ch(side), _ch(uplo), _ch(transa), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B), ldb,
                                 _stream(stream)))


def xgemm_dtrmm(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream=None) -> int:
    return int(lib().xgemm_dtrmm(_ch(side), _ch(uplo), _ch(transa), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B), ldb,
                                 _stream(stream)))


def xgemm_strmm(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream=None) -> int:
    return int(lib().xgemm_strmm(_ch(side), _ch(uplo), _ch(transa), _ch(diag), m, n, alpha, _ptr(A), lda, _ptr(B), ldb,
                                 _stream(stream)))


def xgemm_dpotrf(uplo, n, A, lda, info, stream=None) -> int:
    return int(lib().xgemm_dpotrf(_ch(uplo), n, _ptr(A), lda, _ptr(info), _stream(stream)))


def xgemm_spotrf(uplo, n, A, lda, info, stream=None) -> int:
    return int(lib().xgemm_spotrf(_ch(uplo), n, _ptr(A), lda, _ptr(info), _stream(stream)))


def xgemm_dgetrf(m, n, A, lda, ipiv, info, stream=None) -> int:
    return int(lib().xgemm_dgetrf(m, n, _ptr(A), lda, _ptr(ipiv), _ptr(info), _stream(stream)))


def xgemm_sgetrf(m, n, A, lda, ipiv, info, stream=None) -> int:
    return int(lib().xgemm_sgetrf(m, n, _ptr(A), lda, _ptr(ipiv), _ptr(info), _stream(stream)))


def xgemm_getrf_workspace_bytes() -> int:
    return int(lib().xgemm_getrf_workspace_bytes())


def xgemm_dgetrf_ws(m, n, A, lda, ipiv, info, work, lwork, stream=None) -> int:
    return int(lib().xgemm_dgetrf_ws(m, n, _ptr(A), lda, _ptr(ipiv), _ptr(info), _ptr(work), lwork, _stream(stream)))


def xgemm_sgetrf_ws(m, n, A, lda, ipiv, info, work, lwork, stream=None) -> int:
    return int(lib().xgemm_sgetrf_ws(m, n, _ptr(A), lda, _ptr(ipiv), _ptr(info), _ptr(work), lwork, _stream(stream)))


def xgemm_force_getrf_shared(mode) -> int:
    return int(lib().xgemm_force_getrf_shared(int(mode)))


def xgemm_force_getrf_poll_delay(header_sleeps, row_sleeps) -> int:
    return int(lib().xgemm_force_getrf_poll_delay(int(header_sleeps), int(row_sleeps)))


def xgemm_force_getrf_spin_limit(polls) -> int:
    return int(lib().xgemm_force_getrf_spin_limit(int(polls)))


def xgemm_pack_elems(rows, k) -> int:
    return int(lib().xgemm_pack_elems(int(rows), int(k)))


def _pack_op(name):
    def call(trans, d1, d2, X, ld, Xp, stream=None) -> int:
        return int(getattr(lib(), name)(_ch(trans), d1, d2, _ptr(X), ld, _ptr(Xp), _stream(stream)))
    call.__name__ = name
    return call


xgemm_dpack_a = _pack_op("xgemm_dpack_a")
xgemm_dpack_b = _pack_op("xgemm_dpack_b")
xgemm_spack_a = _pack_op("xgemm_spack_a")
xgemm_spack_b = _pack_op("xgemm_spack_b")


def xgemm_dgemm_packed(m, n, k, alpha, Ap, Bp, beta, C, ldc, stream=None) -> int:
    return int(lib().xgemm_dgemm_packed(m, n, k, alpha, _ptr(Ap), _ptr(Bp), beta, _ptr(C), ldc, _stream(stream)))


def xgemm_sgemm_packed(m, n, k, alpha, Ap, Bp, beta, C, ldc, stream=None) -> int:
    return int(lib().xgemm_sgemm_packed(m, n, k, alpha, _ptr(Ap), _ptr(Bp), beta, _ptr(C), ldc, _stream(stream)))


def xgemm_force_getrf_panel(width) -> int:
    return int(lib().xgemm_force_getrf_panel(int(width)))


def _two_flag_op(name):
    def call(f1, f2, d1, d2, alpha, A, lda, B, ldb, beta, C, ldc, stream=None) -> int:
        return int(getattr(lib(), name)(_ch(f1), _ch(f2), d1, d2, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                                        _stream(stream)))
    call.__name__ = name
    return call


xgemm_dsyr2k = _two_flag_op("xgemm_dsyr2k")   # (uplo, trans, n, k, alpha, A, lda, B, ldb, beta, C, ldc)
xgemm_ssyr2k = _two_flag_op("xgemm_ssyr2k")
xgemm_dsymm = _two_flag_op("xgemm_dsymm")     # (side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc)
xgemm_ssymm = _two_flag_op("xgemm_ssymm")


def xgemm_workspace_bytes() -> int:
    return int(lib().xgemm_workspace_bytes())


def xgemm_workspace_init(work, lwork, stream=None) -> int:
    return int(lib().xgemm_workspace_init(_ptr(work), lwork, _stream(stream)))


def xgemm_dgemm_ws(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, work, lwork, stream=None) -> int:
    return int(lib().xgemm_dgemm_ws(_ch(transa), _ch(transb), m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                    _ptr(C), ldc, _ptr(work), lwork, _stream(stream)))


STATIC_SCRATCH_BYTES = 8192 + (32 << 20)   # XGEMM_STATIC_SCRATCH_BYTES
E_SCRATCH = -1000                           # XGEMM_E_SCRATCH


def xgemm_dgemm_static(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream=None) -> int:
    return int(lib().xgemm_dgemm_static(_ch(transa), _ch(transb), m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                        _ptr(C), ldc, _stream(stream)))


def xgemm_sgemm_ws(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, work, lwork, stream=None) -> int:
    return int(lib().xgemm_sgemm_ws(_ch(transa), _ch(transb), m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                    _ptr(C), ldc, _ptr(work), lwork, _stream(stream)))


def xgemm_dsyrk_ws(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, work, lwork, stream=None) -> int:
    return int(lib().xgemm_dsyrk_ws(_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, beta, _ptr(C), ldc,
                                    _ptr(work), lwork, _stream(stream)))


def xgemm_ssyrk_ws(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, work, lwork, stream=None) -> int:
    return int(lib().xgemm_ssyrk_ws(_ch(uplo), _ch(trans), n, k, alpha, _ptr(A), lda, beta, _ptr(C), ldc,
                                    _ptr(work), lwork, _stream(stream)))


def xgemm_tuning_reset() -> None:
    lib().xgemm_tuning_reset()


def xgemm_release_thread_resources() -> int:
    return int(lib().xgemm_release_thread_resources())


def xgemm_force_split(pieces) -> int:
    return int(lib().xgemm_force_split(int(pieces)))


def xgemm_last_split() -> int:
    return int(lib().xgemm_last_split())


def xgemm_plan(prec, uplo, m, n, k, lwork=0):
    """Returns (variant, pieces per split tile, tiles computed whole) or a negative error code."""
    out = (ctypes.c_int * 3)()
    rc = int(lib().xgemm_plan(_ch(prec), int(uplo), m, n, k, lwork, out))
    return (out[0], out[1], out[2]) if rc == 0 else rc


def _pair(z):
    if z is None:
        return None
    return (ctypes.c_double * 2)(float(z[0]), float(z[1]))


def xgemm_zgemm_split(transa, transb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc,
                      work=None, lwork=0, stream=None) -> int:
    al, be = _pair(alpha), _pair(beta)
    return int(lib().xgemm_zgemm_split(_ch(transa), _ch(transb), m, n, k, al, _ptr(Ar), _ptr(Ai), lda,
                                       _ptr(Br), _ptr(Bi), ldb, be, _ptr(Cr), _ptr(Ci), ldc,
                                       _ptr(work), lwork, _stream(stream)))


def xgemm_zgemm(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, method=0, work=None, lwork=0,
                stream=None) -> int:
    al, be = _pair(alpha), _pair(beta)
    return int(lib().xgemm_zgemm(_ch(transa), _ch(transb), m, n, k, al, _ptr(A), lda, _ptr(B), ldb, be, _ptr(C), ldc,
                                 int(method), _ptr(work), lwork, _stream(stream)))


def xgemm_zgemm_workbytes(m, n, k, method=0) -> int:
    return int(lib().xgemm_zgemm_workbytes(m, n, k, int(method)))


def xgemm_zgemm_worksize(m, n, alpha, beta) -> int:
    return int(lib().xgemm_zgemm_worksize(m, n, _pair(alpha), _pair(beta)))


def xgemm_version() -> str:
    return lib().xgemm_version().decode()


def xgemm_last_kernel_name() -> str:
    return lib().xgemm_last_kernel_name().decode()


def xgemm_force_variant(variant: int) -> int:
    return int(lib().xgemm_force_variant(int(variant)))


def xgemm_variant_name(prec: str, variant: int):
    r = lib().xgemm_variant_name(_ch(prec), int(variant))
    return r.decode() if r else None


def xgemm_mfma_peak_probe(prec, blocks, iters, sink, stream=None) -> int:
    return int(lib().xgemm_mfma_peak_probe(_ch(prec), blocks, iters, _ptr(sink), _stream(stream)))


def xgemm_mfma_layout_probe(prec, out, stream=None) -> int:
    return int(lib().xgemm_mfma_layout_probe(_ch(prec), _ptr(out), _stream(stream)))


def xgemm_hwid_probe(blocks, lds_bytes, out, stream=None) -> int:
    return int(lib().xgemm_hwid_probe(blocks, lds_bytes, _ptr(out), _stream(stream)))


def xgemm_force_potrf_block(order) -> int:
    return int(lib().xgemm_force_potrf_block(int(order)))


def xgemm_force_potrf_panel(width) -> int:
    return int(lib().xgemm_force_potrf_panel(int(width)))


def xgemm_latency_probe(out, sink, iters, stream=None) -> int:
    return int(lib().xgemm_latency_probe(_ptr(out), _ptr(sink), iters, _stream(stream)))


def xgemm_model_outer_product_rate(rate, count) -> float:
    n = len(rate)
    r = (ctypes.c_double * n)(*[float(x) for x in rate])
    c = (ctypes.c_double * n)(*[float(x) for x in count])
    return float(lib().xgemm_model_outer_product_rate(n, r, c))


def xgemm_model_stalled_rate(L, n_dependent, latency) -> float:
    return float(lib().xgemm_model_stalled_rate(L, n_dependent, latency))


def xgemm_model_n_updates(r_total, m_r, n_r, v, r_a, r_r) -> int:
    return int(lib().xgemm_model_n_updates(r_total, m_r, n_r, v, r_a, r_r))


def xgemm_model_predict(prec, variant, transa="N", transb="N"):
    """Returns (status, list of 12 floats); see include/xgemm.h for the fields."""
    out = (ctypes.c_double * 12)()
    rc = int(lib().xgemm_model_predict(_ch(prec), int(variant), _ch(transa), _ch(transb), out))
    return rc, list(out)


def xgemm_model_efficiency(prec, variant):
    """Returns (rc, (measured, model, planner's))."""
    out = (ctypes.c_double * 3)()
    rc = int(lib().xgemm_model_efficiency(_ch(prec), int(variant), out))
    return rc, tuple(out)


def xgemm_model_enumerate(prec, cap=4096):
    """Returns (count, rows): rows is a list of 12-tuples, best predicted utilisation first; see include/xgemm_tuning.h."""
    buf = (ctypes.c_double * (12 * max(cap, 1)))()
    cnt = int(lib().xgemm_model_enumerate(_ch(prec), int(cap), buf))
    if cnt < 0:
        return cnt, None
    n = min(cnt, cap)
    return cnt, [tuple(buf[12 * i + c] for c in range(12)) for i in range(n)]


def xgemm_tile_map(uplo, m, n, mt_m, mt_n, want_tiles=True):
    """Returns (count, tiles): tiles is a list of (tile row, tile column) per workgroup, or None."""
    cnt = int(lib().xgemm_tile_map(int(uplo), m, n, int(mt_m), int(mt_n), None, 0))
    if cnt <= 0 or not want_tiles:
        return cnt, None
    buf = (ctypes.c_int * (2 * cnt))()
    lib().xgemm_tile_map(int(uplo), m, n, int(mt_m), int(mt_n), buf, cnt)
    return cnt, [(buf[2 * b], buf[2 * b + 1]) for b in range(cnt)]
