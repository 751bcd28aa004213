"""Helpers for the GPU parity tests: move seeded numpy operands to the device,
call the library through its C ABI binding, bring C back."""
import numpy as np

import oracle
import synth_inputs as si


def torch_mod():
    import torch
    return torch


def to_dev(X):
    torch = torch_mod()
    return None if X is None else torch.from_numpy(np.ascontiguousarray(X)).cuda()


def run_real(xg, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, expect=0):
    """Run xgemm_{d,s}gemm on copies of the numpy operands; return C after the call."""
    torch = torch_mod()
    f = xg.xgemm_dgemm if C.dtype == np.float64 else xg.xgemm_sgemm
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    rc = f(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc)
    torch.cuda.synchronize()
    assert rc == expect, f"return code {rc}, expected {expect}"
    return dC.cpu().numpy()


def make_operands(rng, ta, tb, m, n, k, pad=(0, 0, 0), dtype=np.float64, kind="uniform", R=8):
    ra, ca = si.operand_shape(ta, m, k)
    rb, cb = si.operand_shape(tb, k, n)
    lda, ldb, ldc = max(ra, 1) + pad[0], max(rb, 1) + pad[1], max(m, 1) + pad[2]
    if kind == "uniform":
        gen = lambda r, c, ld: si.uniform(rng, r, c, ld, dtype)
    elif kind == "normal":
        gen = lambda r, c, ld: si.normal(rng, r, c, ld, dtype)
    else:
        gen = lambda r, c, ld: si.integers(rng, r, c, ld, dtype, R=R)
    return gen(ra, ca, lda), lda, gen(rb, cb, ldb), ldb, gen(m, n, ldc), ldc


def unit_roundoff(dtype):
    return oracle.U64 if np.dtype(dtype) == np.float64 else oracle.U32


def check_full(xg, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, factor=4.0):
    """GPU result against the extended-precision oracle on every element, plus:
    padding rows of C untouched.  Returns the largest err/bound ratio."""
    out = run_real(xg, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc)
    info, Cref, G = oracle.gemm_ext(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc)
    assert info == 0
    nviol, ratio = oracle.bound_violations(out[:, :m], Cref, G, k, unit_roundoff(C.dtype), factor)
    assert nviol == 0, f"{nviol} elements outside the bound (max ratio {ratio}) for {ta}{tb} {m}x{n}x{k}"
    if ldc > m:
        pad_in, pad_out = C[:, m:], out[:, m:]
        assert np.array_equal(pad_in, pad_out, equal_nan=True), "padding rows of C were written"
    return ratio


def check_out_full(out, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, factor=4.0, chunk=1024, label=""):
    """A result already on the host against the extended-precision oracle on EVERY element,
    a block of `chunk` columns of C at a time (op(B) and C cut along n, so that the wide
    reference and magnitude arrays stay small); padding rows of C untouched.  Prints one
    progress line per block.  Returns the largest err/bound ratio."""
    import sys
    import time
    worst = 0.0
    t0 = time.time()
    for j0 in range(0, n, chunk):
        j1 = min(n, j0 + chunk)
        Bc = B[j0:j1] if tb in "Nn" else np.ascontiguousarray(B[:, j0:j1])
        ldbc = ldb if tb in "Nn" else j1 - j0
        info, Cref, G = oracle.gemm_ext(ta, tb, m, j1 - j0, k, alpha, A, lda, Bc, ldbc, beta, C[j0:j1], ldc)
        assert info == 0
        nviol, ratio = oracle.bound_violations(out[j0:j1, :m], Cref, G, k, unit_roundoff(C.dtype), factor)
        assert nviol == 0, f"{nviol} elements outside the bound (max ratio {ratio}) in columns {j0}:{j1} of {ta}{tb} {m}x{n}x{k}"
        worst = max(worst, ratio)
        print(f"  {label} columns {j0}:{j1} of {n} checked, {time.time() - t0:.1f} s", flush=True)
        sys.stdout.flush()
    if ldc > m:
        assert np.array_equal(C[:, m:], out[:, m:], equal_nan=True), "padding rows of C were written"
    return worst


def check_samples(out, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, I, J, factor=4.0):
    info, cref, g = oracle.gemm_samples(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, I, J)
    assert info == 0
    nviol, ratio = oracle.bound_violations(out[J, I], cref, g, k, unit_roundoff(C.dtype), factor)
    assert nviol == 0, f"{nviol} sampled elements outside the bound (max ratio {ratio})"
    return ratio


def run_syrk(xg, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, expect=0):
    """Run xgemm_{d,s}syrk on copies of the numpy operands; return C after the call."""
    torch = torch_mod()
    f = xg.xgemm_dsyrk if C.dtype == np.float64 else xg.xgemm_ssyrk
    dA, dC = to_dev(A), to_dev(C)
    rc = f(uplo, trans, n, k, alpha, dA, lda, beta, dC, ldc)
    torch.cuda.synchronize()
    assert rc == expect, f"return code {rc}, expected {expect}"
    return dC.cpu().numpy()


def make_syrk_operands(rng, trans, n, k, pad=(0, 0), dtype=np.float64, kind="uniform", R=8):
    ra, ca = (n, k) if trans == "N" else (k, n)
    lda, ldc = max(ra, 1) + pad[0], max(n, 1) + pad[1]
    if kind == "uniform":
        gen = lambda r, c, ld: si.uniform(rng, r, c, ld, dtype)
    else:
        gen = lambda r, c, ld: si.integers(rng, r, c, ld, dtype, R=R)
    return gen(ra, ca, lda), lda, gen(n, n, ldc), ldc


def check_syrk_full(xg, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, factor=4.0):
    """GPU triangle against the extended-precision oracle on every element of the
    triangle; everything else in the buffer (other triangle, padding rows) must be
    bit-identical to the input.  Returns the largest err/bound ratio."""
    out = run_syrk(xg, uplo, trans, n, k, alpha, A, lda, beta, C, ldc)
    info, Cref, G = oracle.syrk_ext(uplo, trans, n, k, alpha, A, lda, beta, C, ldc)
    assert info == 0
    mask = oracle.triangle_mask(uplo, n)
    got = np.where(mask, out[:, :n], 0).astype(out.dtype)
    nviol, ratio = oracle.bound_violations(got, Cref, G, k, unit_roundoff(C.dtype), factor)
    assert nviol == 0, f"{nviol} elements outside the bound (max ratio {ratio}) for {uplo}{trans} {n}x{k}"
    keep = np.ones(C.shape, dtype=bool)
    keep[:, :n] = ~mask
    assert np.array_equal(out[keep], C[keep], equal_nan=True), "elements outside the triangle were written"
    return ratio
