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


@pytest.fixture(autouse=True)
def _panel_by_order():
    xg.xgemm_force_potrf_panel(-1)
    xg.xgemm_force_potrf_block(-1)
    yield
    xg.xgemm_force_potrf_panel(-1)
    xg.xgemm_force_potrf_block(-1)


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
    # relative, except for entries that cancel to far below the terms they are summed from: those carry
    # the absolute rounding error of the terms (the order of the sums differs between the two routes)
    assert np.allclose(got, want, rtol=tol, atol=1e-3 * tol * float(np.max(np.abs(want))))
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
    """Orders 1..64 are one launch of the one-wave block kernel each, orders up to 128 (fp32: 256) one
    launch of the kernel with a wave per 64x64 block (ragged last panels and tiles, blocks that lie
    partly or wholly beyond the order, the careful route for a panel of fewer than four columns);
    above that the solve and update kernels join in.  Integer factors recovered exactly, three times each."""
    rng = si.rng_for(175, "LU".index(uplo))
    for n in range(1, 257):
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


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("uplo", "LU")
def test_look_ahead_sweep_with_small_panels(dtype, uplo):
    """The panel sweep with look-ahead on a second stream (the form large orders take), forced onto small
    orders so that the oracle can check every element: two panels, many panels, a ragged last panel, a
    last panel of one column, panels narrower and wider than the diagonal-block kernel's order."""
    rng = si.rng_for(175, 0 if uplo == "L" else 1)
    for n, W, pad in [(517, 128, 2), (1000, 192, 0), (700, 64, 1), (300, 256, 0), (257, 256, 3), (640, 320, 0), (130, 40, 1)]:
        A = si.spd(rng, n, n + pad, dtype, uplo)
        assert xg.xgemm_force_potrf_panel(W) == 0
        F, info = run_potrf(uplo, n, A, n + pad)
        assert info == 0
        assert np.array_equal(np.isnan(F), np.isnan(A)), "something outside the triangle was written"
        rinfo, R, G = oracle.potrf_resid(uplo, n, A, n + pad, F, n + pad)
        assert rinfo == 0
        bound = 4.0 * n * unit_roundoff(dtype) * G
        assert np.all(np.abs(R) <= bound), f"{uplo} n={n} W={W}: max ratio {float(np.max(np.abs(R) / np.maximum(bound, 1e-300)))}"
        # the same run again gives the same bits (the two streams are ordered by events, not by luck)
        F2, _ = run_potrf(uplo, n, A, n + pad)
        assert np.array_equal(F, F2, equal_nan=True)
        # and agrees with the recursion on one stream to rounding
        assert xg.xgemm_force_potrf_panel(0) == 0
        F1, info1 = run_potrf(uplo, n, A, n + pad)
        tol = 16 * n * unit_roundoff(dtype)
        mask = oracle.triangle_mask(uplo, n)
        assert info1 == 0 and np.allclose(F[:, :n][mask], F1[:, :n][mask], rtol=tol, atol=tol)


@pytest.mark.parametrize("uplo", "LU")
def test_look_ahead_sweep_integer_factor_and_failure_report(uplo):
    rng = si.rng_for(176, 0)
    n, R = 300, 3
    L0 = np.tril(rng.integers(-R, R + 1, size=(n, n)), -1).astype(np.int64)
    L0[np.arange(n), np.arange(n)] = 2 ** rng.integers(0, 3, size=n)
    A = np.full((n, n + 1), np.nan)
    A[:, :n] = (L0 @ L0.T).astype(np.float64)
    si._mask_triangle(A, n, uplo, False, np.nan)
    assert xg.xgemm_force_potrf_panel(64) == 0
    F, info = run_potrf(uplo, n, A, n + 1)
    mask = oracle.triangle_mask(uplo, n)
    assert info == 0 and np.array_equal(F[:, :n][mask], (L0.T if uplo == "L" else L0)[mask].astype(np.float64))
    # the first failing minor is reported whichever panel it falls into
    for bad in (10, 64, 131, 299):
        B = si.spd(rng, n, n, np.float64, uplo)
        B[bad, bad] = -1.0
        _, info = run_potrf(uplo, n, B, n)
        assert info == bad + 1


def test_look_ahead_sweep_is_the_default_for_large_orders_and_graph_safe():
    """n = 3200 takes the sweep by itself; captured in a graph after one eager call, every replay gives the eager bits."""
    torch = torch_mod()
    rng = si.rng_for(177, 0)
    n = 3200
    S0 = to_dev(si.spd(rng, n, n, np.float64, "L", sentinel=0.0))
    S = S0.clone()
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert xg.xgemm_dpotrf("L", n, S, n, info) == 0
    torch.cuda.synchronize()
    want = S.clone()
    assert int(info.item()) == 0
    assert xg.xgemm_force_potrf_panel(0) == 0
    S.copy_(S0)
    assert xg.xgemm_dpotrf("L", n, S, n, info) == 0
    torch.cuda.synchronize()
    assert not torch.equal(S, want), "the default at this order was meant to differ from the recursion (another order of sums)"
    assert torch.allclose(torch.tril(S), torch.tril(want), rtol=1e-10, atol=1e-10)
    assert xg.xgemm_force_potrf_panel(-1) == 0
    graph = torch.cuda.CUDAGraph()
    S.copy_(S0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        assert xg.xgemm_dpotrf("L", n, S, n, info) == 0
    for rep in range(3):
        S.copy_(S0)
        info.fill_(7)
        scratch = torch.rand(512, 512, device="cuda") @ torch.rand(512, 512, device="cuda")
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(S, want), f"replay {rep} differs from the eager run"
        assert int(info.item()) == 0
        del scratch


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("uplo", "LU")
@pytest.mark.parametrize("block", [64, 128, 256])
def test_diagonal_block_kernels_of_every_size(dtype, uplo, block):
    """The same factorisations with diagonal blocks of up to 64, 128 and 256 handed to one workgroup
    (one wave; a wave per 64x64 block, three or ten of them): residual bound on every element, the first
    failing minor wherever it falls (in a diagonal block's fast or careful route, first or last block
    column), and pivots so small or large that every panel takes the careful route."""
    assert xg.xgemm_force_potrf_block(block) == 0
    rng = si.rng_for(178, block)
    u = unit_roundoff(dtype)
    for n in (100, 128, 129, 200, 256, 300):
        A = si.spd(rng, n, n + 1, dtype, uplo)
        F, info = run_potrf(uplo, n, A, n + 1)
        assert info == 0
        assert np.array_equal(np.isnan(F), np.isnan(A)), "something outside the triangle was written"
        rinfo, R, G = oracle.potrf_resid(uplo, n, A, n + 1, F, n + 1)
        assert rinfo == 0 and np.all(np.abs(R) <= 4.0 * n * u * G), f"n={n}"
        F2, _ = run_potrf(uplo, n, A, n + 1)
        assert np.array_equal(F, F2, equal_nan=True)
    n = 256
    for bad in (0, 3, 63, 64, 70, 127, 128, 130, 200, 255):
        B = si.spd(rng, n, n, dtype, uplo)
        B[bad, bad] = -1.0
        _, info = run_potrf(uplo, n, B, n)
        assert info == bad + 1, f"bad pivot {bad}"
    shift = -780 if dtype == np.float64 else -110
    A = si.spd(rng, n, n, dtype, uplo)
    F1, info1 = run_potrf(uplo, n, A, n)
    F2, info2 = run_potrf(uplo, n, np.ldexp(A, shift).astype(dtype), n)
    assert info1 == 0 and info2 == 0
    mask = oracle.triangle_mask(uplo, n)
    got = np.ldexp(F2[:, :n][mask].astype(np.float64), -shift // 2)
    want = F1[:, :n][mask].astype(np.float64)
    assert np.allclose(got, want, rtol=16 * n * u, atol=1e-3 * 16 * n * u * float(np.max(np.abs(want))))


def test_look_ahead_sweep_on_a_stream_of_the_callers():
    """The sweep forks from and joins whatever stream it is given: on a stream of the caller's, with work
    of the caller's before and after it on that stream and no synchronisation in between, it gives the
    bits of the call on the default stream."""
    torch = torch_mod()
    rng = si.rng_for(179, 0)
    n = 3200
    S0 = to_dev(si.spd(rng, n, n, np.float64, "U", sentinel=0.0))
    S = S0.clone()
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert xg.xgemm_dpotrf("U", n, S, n, info) == 0
    torch.cuda.synchronize()
    want = S.clone()
    side = torch.cuda.Stream()
    for rep in range(2):
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            S.copy_(S0)                                        # the factorisation must wait for this copy ...
            assert xg.xgemm_dpotrf("U", n, S, n, info, stream=side) == 0
            got = S.clone()                                    # ... and this copy for the factorisation
        side.synchronize()
        assert torch.equal(got, want), f"run {rep}"
        assert int(info.item()) == 0


def test_thread_resources_can_be_released_and_come_back():
    """The sweep's streams and events are kept per thread and device; releasing them (also when there are
    none, and twice in a row) is harmless, and the next sweep creates them again and gives the same bits."""
    assert xg.xgemm_release_thread_resources() == 0           # whatever earlier tests left, or nothing
    assert xg.xgemm_release_thread_resources() == 0
    rng = si.rng_for(179, 1)
    n = 900
    A = si.spd(rng, n, n + 1, np.float64, "L")
    assert xg.xgemm_force_potrf_panel(128) == 0
    F1, info1 = run_potrf("L", n, A, n + 1)
    assert xg.xgemm_release_thread_resources() == 0
    F2, info2 = run_potrf("L", n, A, n + 1)
    assert info1 == 0 and info2 == 0 and np.array_equal(F1, F2, equal_nan=True)
    rinfo, R, G = oracle.potrf_resid("L", n, A, n + 1, F2, n + 1)
    assert rinfo == 0 and np.all(np.abs(R) <= 4.0 * n * oracle.U64 * G)
