"""GPU parity of the explicit packing and of the product on packed operands.

The packed layout is part of the interface (include/xgemm.h), so it is checked element by element against the
formula stated there, padding included; the product on two packed buffers is checked against the CPU oracle of
the plain product on the unpacked operands, to the same bound as the plain GPU product."""
import itertools

import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import make_operands, to_dev, torch_mod, unit_roundoff

pytestmark = pytest.mark.gpu

PW, KR = 256, 32


def op_of(X, trans, stored_rows):
    """op(X) as a numpy matrix from the column-major storage (array of shape (stored_cols, ld))."""
    V = si.view(X, stored_rows)                          # (stored_rows, stored_cols)
    return V if trans == "N" else V.T


def expected_packed(M):
    """M: (rows, k) matrix, rows being the op's m (or n) index.  The documented layout, as a flat array."""
    rows, k = M.shape
    rpad, kpad = -(-rows // PW) * PW, -(-k // KR) * KR
    out = np.zeros(rpad * kpad, dtype=M.dtype)
    i, p = np.meshgrid(np.arange(rows), np.arange(k), indexing="ij")
    out[(i // PW) * PW * kpad + p * PW + i % PW] = M
    return out


def pack(side, trans, d1, d2, X, ld):
    torch = torch_mod()
    dt = X.dtype
    f = {("a", np.float64): xg.xgemm_dpack_a, ("b", np.float64): xg.xgemm_dpack_b,
         ("a", np.float32): xg.xgemm_spack_a, ("b", np.float32): xg.xgemm_spack_b}[(side, dt.type)]
    rows, k = (d1, d2) if side == "a" else (d2, d1)
    n_el = xg.xgemm_pack_elems(rows, k)
    buf = torch.full((max(n_el, 1),), float("nan"), dtype=torch.float64 if dt == np.float64 else torch.float32, device="cuda")
    rc = f(trans, d1, d2, to_dev(X), ld, buf)
    torch.cuda.synchronize()
    assert rc == 0, rc
    return buf, n_el


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("side,trans", list(itertools.product("ab", "NT")))
def test_layout_is_the_documented_one(dtype, side, trans):
    rng = si.rng_for(310, "abNT".index(side) * 2 + "NT".index(trans))
    for (rows, k), pad in zip([(300, 70), (513, 33), (1, 1), (256, 32), (64, 1000), (1000, 257)], itertools.cycle([0, 5])):
        # op(A) is rows x k; op(B) is k x rows
        d1, d2 = (rows, k) if side == "a" else (k, rows)
        sr, sc = (d1, d2) if trans == "N" else (d2, d1)      # stored shape
        ld = sr + pad
        X = si.uniform(rng, sr, sc, ld, dtype)
        buf, n_el = pack(side, trans, d1, d2, X, ld)
        assert n_el == (-(-rows // PW) * PW) * (-(-k // KR) * KR)
        O = op_of(X, trans, sr)                              # d1 x d2
        M = O if side == "a" else O.T                        # (rows, k)
        got = buf.cpu().numpy()[:n_el]
        want = expected_packed(np.ascontiguousarray(M))
        assert np.array_equal(got, want), f"{side}{trans} {rows}x{k}: {int(np.sum(got != want))} elements differ (NaN = not written)"


def run_packed(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc):
    torch = torch_mod()
    Ap, _ = pack("a", ta, m, k, A, lda)
    Bp, _ = pack("b", tb, k, n, B, ldb)
    dC = to_dev(C)
    f = xg.xgemm_dgemm_packed if C.dtype == np.float64 else xg.xgemm_sgemm_packed
    rc = f(m, n, k, alpha, Ap, Bp, beta, dC, ldc)
    torch.cuda.synchronize()
    assert rc == 0, rc
    return dC.cpu().numpy()


def check(ta, tb, m, n, k, alpha, beta, A, lda, B, ldb, C, ldc, factor=4.0):
    out = run_packed(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc)
    info, Cref, G = oracle.gemm_ext(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc)
    assert info == 0
    nviol, ratio = oracle.bound_violations(out[:, :m], Cref, G, k, unit_roundoff(C.dtype), factor)
    assert nviol == 0, f"{nviol} elements outside the bound (max ratio {ratio}) for {ta}{tb} {m}x{n}x{k}"
    if ldc > m:
        assert np.array_equal(C[:, m:], out[:, m:], equal_nan=True), "padding rows of C were written"
    return out


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("ta,tb", list(itertools.product("NT", "NT")))
def test_packed_product_against_oracle(dtype, ta, tb):
    rng = si.rng_for(311, "NT".index(ta) * 2 + "NT".index(tb))
    shapes = [(129, 65, 33), (1000, 700, 300), (257, 513, 16), (1, 1, 1), (64, 64, 8), (300, 2, 1025), (1536, 1024, 512)]
    for (m, n, k), pad, (alpha, beta) in zip(shapes, itertools.cycle([(0, 0, 0), (3, 5, 7)]),
                                             itertools.cycle([(1.5, -0.5), (1.0, 0.0), (-2.0, 1.0)])):
        A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad, dtype)
        check(ta, tb, m, n, k, alpha, beta, A, lda, B, ldb, C, ldc)


def test_integer_data_bit_exact_and_beta_zero_ignores_nan():
    rng = si.rng_for(312, 0)
    m, n, k = 700, 500, 333
    A, lda, B, ldb, C, ldc = make_operands(rng, "T", "N", m, n, k, (1, 2, 3), np.float64, kind="int")
    C[:, :m] = np.nan                                            # beta = 0: C is not read
    out = run_packed("T", "N", m, n, k, 2.0, A, lda, B, ldb, 0.0, C, ldc)
    want = np.zeros_like(C)
    assert oracle.gemm_work("T", "N", m, n, k, 2.0, A, lda, B, ldb, 0.0, want, ldc) == 0
    assert np.array_equal(out[:, :m], want[:, :m])


def test_a_packed_operand_serves_several_products():
    torch = torch_mod()
    rng = si.rng_for(313, 0)
    m, k = 900, 260
    A = si.uniform(rng, m, k, m, np.float64)
    Ap, _ = pack("a", "N", m, k, A, m)
    for n in (1, 130, 777):
        B = si.uniform(rng, k, n, k + 1, np.float64)
        C = si.uniform(rng, m, n, m, np.float64)
        Bp, _ = pack("b", "N", k, n, B, k + 1)
        dC = to_dev(C)
        assert xg.xgemm_dgemm_packed(m, n, k, 1.0, Ap, Bp, 1.0, dC, m) == 0
        torch.cuda.synchronize()
        info, Cref, G = oracle.gemm_ext("N", "N", m, n, k, 1.0, A, m, B, k + 1, 1.0, C, m)
        nviol, ratio = oracle.bound_violations(dC.cpu().numpy()[:, :m], Cref, G, k, oracle.U64, 4.0)
        assert info == 0 and nviol == 0, (n, ratio)


def test_degenerate_calls():
    torch = torch_mod()
    C = torch.full((6,), 3.0, dtype=torch.float64, device="cuda")
    assert xg.xgemm_dgemm_packed(2, 3, 0, 1.0, None, None, 0.5, C, 2) == 0      # k = 0: C := beta C
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy(), np.full(6, 1.5))
    assert xg.xgemm_dgemm_packed(2, 3, 5, 0.0, None, None, 2.0, C, 2) == 0      # alpha = 0: operands not read
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy(), np.full(6, 3.0))
    assert xg.xgemm_dgemm_packed(0, 3, 5, 1.0, None, None, 2.0, None, 1) == 0
    assert xg.xgemm_dpack_a("N", 0, 5, None, 1, None) == 0
