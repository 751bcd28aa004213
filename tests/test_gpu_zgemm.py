"""GPU parity of the interleaved complex GEMM (4m and 3m) against the complex
oracle.  The oracle works on split planes; the interleaved operands are taken
apart with numpy slicing (layout only) before it is called.

Bounds per plane, u = 2^-53: 4m: 8 k u G_plane, G_plane the sum of magnitudes of
the real products entering that plane (two chained real GEMMs of depth k).  The fused
form (method 2) is one real GEMM of depth 2k over the same products (alpha folded into
the expanded A, which costs two roundings per entry): the same bound.
3m: the imaginary part is T3 - T1 - T2 with T3 = (Ar + Ai)(Br + Bi), whose
magnitudes are those of both planes together: 8 k u (G_re + G_im) for both."""
import itertools

import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import to_dev, torch_mod

pytestmark = pytest.mark.gpu


def zmat(rng, rows, cols, ld, kind="uniform", R=8):
    """Interleaved complex matrix as float64 array of shape (cols, 2*ld) plus its planes."""
    gen = (lambda: si.uniform(rng, rows, cols, ld)) if kind == "uniform" else (lambda: si.integers(rng, rows, cols, ld, R=R))
    re, im = gen(), gen()
    Z = np.empty((cols, 2 * ld))
    Z[:, 0::2], Z[:, 1::2] = re, im
    return Z, re, im


def operands(rng, ta, tb, m, n, k, pad=(0, 0, 0), kind="uniform"):
    ra, ca = si.operand_shape("N" if ta == "N" else "T", m, k)
    rb, cb = si.operand_shape("N" if tb == "N" else "T", k, n)
    lda, ldb, ldc = max(ra, 1) + pad[0], max(rb, 1) + pad[1], max(m, 1) + pad[2]
    return zmat(rng, ra, ca, lda, kind), lda, zmat(rng, rb, cb, ldb, kind), ldb, zmat(rng, m, n, ldc, kind), ldc


def run(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, method):
    torch = torch_mod()
    lw = xg.xgemm_zgemm_workbytes(m, n, k, method)
    work = torch.empty(max(lw, 16), dtype=torch.uint8, device="cuda")
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    assert xg.xgemm_zgemm(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc, method, work, lw) == 0
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    return out[:, 0::2], out[:, 1::2]


@pytest.mark.parametrize("method", [0, 1, 2])
@pytest.mark.parametrize("ta,tb", list(itertools.product("NTC", "NTC")))
def test_small_full_check(ta, tb, method):
    rng = si.rng_for(150, method)
    m, n, k = 150, 131, 77
    for alpha, beta in [((1.0, 0.0), (0.0, 0.0)), ((0.75, -1.25), (0.5, 2.0)), ((0.0, 1.0), (1.0, 0.0))]:
        (A, Ar, Ai), lda, (B, Br, Bi), ldb, (C, Cr, Ci), ldc = operands(rng, ta, tb, m, n, k, (2, 4, 6))
        if beta == (0.0, 0.0):
            C[:, : 2 * m] = np.nan                     # beta == 0: C is write-only
        Or, Oi = run(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, method)
        info, Rr, Ri, Gr, Gi = oracle.zgemm_split_ext(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc)
        assert info == 0
        for O, R, G, P in ((Or, Rr, Gr, Cr), (Oi, Ri, Gi, Ci)):
            Gb = Gr + Gi if method == 1 else G
            nviol, ratio = oracle.bound_violations(O[:, :m], R, Gb, k, oracle.U64, factor=8.0)
            assert nviol == 0, (ta, tb, method, alpha, beta, ratio)
            assert np.array_equal(O[:, m:], P[:, m:], equal_nan=True), "padding of C was written"


@pytest.mark.parametrize("method", [0, 1, 2])
def test_gaussian_integers_bit_exact(method):
    rng = si.rng_for(151, method)
    m, n, k = 200, 260, 129
    for (ta, tb), (alpha, beta) in zip([("N", "N"), ("C", "T"), ("T", "C")],
                                       [((1.0, 0.0), (0.0, 0.0)), ((2.0, 0.0), (-1.0, 0.0)), ((2.0, -1.0), (1.0, 3.0))]):
        (A, Ar, Ai), lda, (B, Br, Bi), ldb, (C, Cr, Ci), ldc = operands(rng, ta, tb, m, n, k, (0, 2, 0), "int")
        Or, Oi = run(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, method)
        Wr, Wi = Cr.copy(), Ci.copy()
        assert oracle.zgemm_split_work(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Wr, Wi, ldc) == 0
        assert np.array_equal(Or, Wr, equal_nan=True) and np.array_equal(Oi, Wi, equal_nan=True)


def test_scalar_paths():
    rng = si.rng_for(152, 0)
    m, n, k = 70, 50, 30
    (A, Ar, Ai), lda, (B, Br, Bi), ldb, (C, Cr, Ci), ldc = operands(rng, "N", "N", m, n, k, (1, 1, 1))
    torch = torch_mod()
    # alpha == 0: A, B and the workspace are not needed; C := beta C
    dC = to_dev(C)
    assert xg.xgemm_zgemm("N", "N", m, n, k, (0.0, 0.0), None, lda, None, ldb, (0.5, 2.0), dC, ldc, 0, None, 0) == 0
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    info, Rr, Ri, Gr, Gi = oracle.zgemm_split_ext("N", "N", m, n, k, (0.0, 0.0), None, None, lda, None, None, ldb,
                                                  (0.5, 2.0), Cr, Ci, ldc)
    assert info == 0
    for O, R, G in ((out[:, 0::2], Rr, Gr), (out[:, 1::2], Ri, Gi)):
        assert oracle.bound_violations(O[:, :m], R, G, 1, oracle.U64, 8.0)[0] == 0
    # k == 0 with beta == 1: nothing happens
    dC = to_dev(C)
    assert xg.xgemm_zgemm("N", "N", m, n, 0, (1.0, 0.0), None, m, None, 1, (1.0, 0.0), dC, ldc, 1, None, 0) == 0
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C, equal_nan=True)


@pytest.mark.parametrize("method", [0, 1, 2])
def test_4096_sampled(method):
    nsz = 4096
    rng = si.rng_for(153, method)
    (A, Ar, Ai), lda, (B, Br, Bi), ldb, (C, Cr, Ci), ldc = operands(rng, "N", "C", nsz, nsz, nsz)
    alpha, beta = (1.0, -0.5), (0.5, 0.25)
    Or, Oi = run("N", "C", nsz, nsz, nsz, alpha, A, lda, B, ldb, beta, C, ldc, method)
    I, J = si.sample_indices(rng, nsz, nsz, 2, 2, 4096)
    info, rr, ri, gr, gi = oracle.zgemm_split_samples("N", "C", nsz, nsz, nsz, alpha, Ar, Ai, lda, Br, Bi, ldb, beta,
                                                      Cr, Ci, ldc, I, J)
    assert info == 0
    for O, r, g in ((Or, rr, gr), (Oi, ri, gi)):
        gb = gr + gi if method == 1 else g
        nviol, ratio = oracle.bound_violations(O[J, I], r, gb, nsz, oracle.U64, factor=8.0)
        assert nviol == 0, ratio


def test_fused_ragged_shapes_and_complex_beta():
    """Method 2 on shapes that leave partial panels and slabs in both packed operands, with a complex beta
    (the pass over C of its own) and with beta = 0 on a C full of NaN."""
    rng = si.rng_for(154, 0)
    for (m, n, k), (ta, tb), (alpha, beta) in zip([(129, 257, 17), (1, 1, 1), (300, 70, 130), (64, 513, 33)],
                                                  [("N", "N"), ("C", "C"), ("T", "N"), ("N", "C")],
                                                  [((1.0, 0.0), (0.0, 0.0)), ((0.5, -2.0), (0.25, 1.5)),
                                                   ((-1.0, 0.0), (1.0, 0.0)), ((0.0, 1.0), (0.0, -1.0))]):
        (A, Ar, Ai), lda, (B, Br, Bi), ldb, (C, Cr, Ci), ldc = operands(rng, ta, tb, m, n, k, (1, 0, 3))
        if beta == (0.0, 0.0):
            C[:, : 2 * m] = np.nan
        Or, Oi = run(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, 2)
        info, Rr, Ri, Gr, Gi = oracle.zgemm_split_ext(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc)
        assert info == 0
        for O, R, G, P in ((Or, Rr, Gr, Cr), (Oi, Ri, Gi, Ci)):
            nviol, ratio = oracle.bound_violations(O[:, :m], R, G, k, oracle.U64, factor=8.0)
            assert nviol == 0, (m, n, k, ta, tb, ratio)
            assert np.array_equal(O[:, m:], P[:, m:], equal_nan=True), "padding of C was written"
