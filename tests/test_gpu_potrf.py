"""GPU parity of the Cholesky driver against the CPU oracle: the componentwise
residual |A - L L^T| <= 4 n u |L||L|^T evaluated by the oracle in extended
precision (the bound any ordering of the sums satisfies), agreement with the
oracle's factor on well-conditioned input, integer factors bit for bit, the
other triangle untouched, failure reporting."""
import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import to_dev, torch_mod, unit_roundoff

pytestmark = pytest.mark.gpu


def run_potrf(uplo, n, A, lda):
    torch = torch_mod()
    f = xg.xgemm_dpotrf if A.dtype == np.float64 else xg.xgemm_spotrf
    dA = to_dev(A)
    dinfo = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    assert f(uplo, n, dA, lda, dinfo) == 0
    torch.cuda.synchronize()
    return dA.cpu().numpy(), int(dinfo.item())


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("uplo", "LU")
def test_sizes_from_one_block_to_several_levels(dtype, uplo):
    rng = si.rng_for(170, 0 if uplo == "L" else 1)
    for n, pad in [(1, 0), (37, 3), (64, 0), (65, 1), (200, 5), (517, 2), (1000, 0)]:
        A = si.spd(rng, n, n + pad, dtype, uplo)
        F, info = run_potrf(uplo, n, A, n + pad)
        assert info == 0
        assert np.array_equal(np.isnan(F), np.isnan(A)), "something outside the triangle was written"
        rinfo, R, G = oracle.potrf_resid(uplo, n, A, n + pad, F, n + pad)
        assert rinfo == 0
        bound = 4.0 * n * unit_roundoff(dtype) * G
        assert np.all(np.abs(R) <= bound), f"{uplo} n={n}: max ratio {float(np.max(np.abs(R) / np.maximum(bound, 1e-300)))}"
        want = A.copy()
        assert oracle.potrf(uplo, n, want, n + pad) == 0
        tol = 16 * n * unit_roundoff(dtype)
        mask = oracle.triangle_mask(uplo, n)
        assert np.allclose(F[:, :n][mask], want[:, :n][mask], rtol=tol, atol=tol)


@pytest.mark.parametrize("dtype,shift", [(np.float64, -780), (np.float32, -110), (np.float64, 900), (np.float32, 100)])
def test_pivots_far_from_one(dtype, shift):
    """Pivots near the bottom of the normal range (where the block kernel leaves its
    reciprocal square root estimate for the library's square root) and near the top:
    scaling A by a power of four scales the factor by a power of two, exactly."""
    rng = si.rng_for(174, shift)
    n = 150
    A = si.spd(rng, n, n, dtype, "L")
    F1, info1 = run_potrf("L", n, A, n)
    F2, info2 = run_potrf("L", n, np.ldexp(A, shift).astype(dtype), n)
    assert info1 == 0 and info2 == 0
    mask = oracle.triangle_mask("L", n)
    got = np.ldexp(F2[:, :n][mask].astype(np.float64), -shift // 2)
    want = F1[:, :n][mask].astype(np.float64)
    tol = 16 * n * unit_roundoff(dtype)
    assert np.allclose(got, want, rtol=tol, atol=0.0)
    rinfo, R, G = oracle.potrf_resid("L", n, np.ldexp(A, shift).astype(dtype), n, F2, n)
    assert rinfo == 0 and np.all(np.abs(R) <= 4.0 * n * unit_roundoff(dtype) * G)


@pytest.mark.parametrize("dtype,R", [(np.float64, 3), (np.float32, 1)])
@pytest.mark.parametrize("uplo", "LU")
def test_integer_factor_bit_exact(dtype, R, uplo):
    rng = si.rng_for(171, 0)
    n = 300
    L0 = np.tril(rng.integers(-R, R + 1, size=(n, n)), -1).astype(np.int64)
    L0[np.arange(n), np.arange(n)] = 2 ** rng.integers(0, 3, size=n)
    M = L0 @ L0.T
    A = np.full((n, n + 1), np.nan, dtype=dtype)
    A[:, :n] = M.astype(dtype)
    si._mask_triangle(A, n, uplo, False, np.nan)
    F, info = run_potrf(uplo, n, A, n + 1)
    want = A.copy()
    assert oracle.potrf(uplo, n, want, n + 1) == 0
    assert info == 0 and np.array_equal(F, want, equal_nan=True)
    mask = oracle.triangle_mask(uplo, n)
    assert np.array_equal(F[:, :n][mask], (L0.T if uplo == "L" else L0)[mask].astype(dtype))


def test_not_positive_definite_is_reported():
    rng = si.rng_for(172, 0)
    n = 200
    A = si.spd(rng, n, n, np.float64, "L")
    A[130, 130] = -1.0                    # the leading minor of order 131 is the first that fails
    F, info = run_potrf("L", n, A, n)
    assert info == 131
    want = A.copy()
    assert oracle.potrf("L", n, want, n) == 131
    # an empty problem clears info
    torch = torch_mod()
    dinfo = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    assert xg.xgemm_dpotrf("U", 0, None, 1, dinfo) == 0
    torch.cuda.synchronize()
    assert int(dinfo.item()) == 0


@pytest.mark.parametrize("dtype,uplo,n", [(np.float64, "L", 8192), (np.float64, "U", 4096), (np.float32, "L", 8192)])
def test_full_size_sampled_residual(dtype, uplo, n):
    rng = si.rng_for(173, n)
    ld = n + 8
    A = si.spd(rng, n, ld, dtype, uplo)
    F, info = run_potrf(uplo, n, A, ld)
    assert info == 0
    I, J = si.sample_indices(rng, n, n, 3, 3, 8192)
    lo = (I >= J) if uplo == "L" else (I <= J)
    I, J = np.where(lo, I, J), np.where(lo, J, I)
    rinfo, R, G = oracle.potrf_resid(uplo, n, A, ld, F, ld, I, J)
    assert rinfo == 0 and np.all(np.abs(R) <= 4.0 * n * unit_roundoff(dtype) * G)
    # a band of columns in full: outside the triangle nothing changed
    for j0 in (0, n // 2, n - 100):
        assert np.array_equal(np.isnan(F[j0:j0 + 100]), np.isnan(A[j0:j0 + 100]))


@pytest.mark.parametrize("dtype,R", [(np.float64, 3), (np.float32, 1)])
@pytest.mark.parametrize("uplo", "LU")
def test_every_order_of_a_single_diagonal_block_bit_exact(dtype, R, uplo):
    """Orders 1..64 are one launch of the block kernel each (ragged last panels and tiles, the
    careful route for a panel of fewer than four columns); then every multiple of 16 up to 256,
    where the solve and update kernels join in.  Integer factors recovered exactly, three times each."""
    rng = si.rng_for(175, "LU".index(uplo))
    for n in list(range(1, 65)) + list(range(80, 257, 16)):
        L0 = np.tril(rng.integers(-R, R + 1, size=(n, n)), -1).astype(np.int64)
        L0[np.arange(n), np.arange(n)] = 2 ** rng.integers(0, 3, size=n)
        A = np.full((n, n + 1), np.nan, dtype=dtype)
        A[:, :n] = (L0 @ L0.T).astype(dtype)
        si._mask_triangle(A, n, uplo, False, np.nan)
        mask = oracle.triangle_mask(uplo, n)
        for rep in range(3):
            F, info = run_potrf(uplo, n, A, n + 1)
            assert info == 0, f"order {n}, run {rep}"
            assert np.array_equal(F[:, :n][mask], (L0.T if uplo == "L" else L0)[mask].astype(dtype)), f"order {n}, run {rep}"
