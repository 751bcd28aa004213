"""GPU parity: the HIP library (through its C ABI) against the CPU oracle.

Floating point: |C_gpu - C_ref|_ij <= 4 k u (|alpha||A||B| + |beta||C|)_ij with
u = 2^-53 (fp64) / 2^-24 (fp32), C_ref from the extended-precision oracle.
Integer-valued inputs: bit-exact.  The complex routine chains two real GEMMs
per plane, so its factor is 8 (two accumulations of depth k, each within 4ku).
"""
import itertools

import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import (check_full, check_out_full, check_samples, make_operands, run_real, to_dev, torch_mod, unit_roundoff)

pytestmark = pytest.mark.gpu

TRANS = ["N", "T"]
DTYPES = [np.float64, np.float32]


def nvariants(prec):
    n = 0
    while xg.xgemm_variant_name(prec, n) is not None:
        n += 1
    return n


@pytest.fixture(autouse=True)
def _auto_variant():
    xg.xgemm_force_variant(-1)
    yield
    xg.xgemm_force_variant(-1)


# --------------------------------------------------------------------------
# accumulator register layout assumed by the kernels
# --------------------------------------------------------------------------
@pytest.mark.parametrize("prec", ["d", "s"])
def test_mfma_accumulator_layout(prec):
    torch = torch_mod()
    R = 4 if prec == "d" else 16
    out = torch.full((64 * R,), -1, dtype=torch.int32, device="cuda")
    assert xg.xgemm_mfma_layout_probe(prec, out) == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(64, R)
    lane = np.arange(64)[:, None]
    r = np.arange(R)[None, :]
    if prec == "d":
        row, col = (lane >> 4) + 4 * r, (lane & 15) + 0 * r
    else:
        row, col = (r & 3) + 4 * (lane >> 5) + 8 * (r >> 2), (lane & 31) + 0 * r
    print("layout", prec, got[:4].tolist())
    assert np.array_equal(got, 256 * row + col)


def test_workgroups_are_dealt_round_robin_to_xcds():
    """The tile order assumes that workgroups are dealt round-robin to the 8 XCDs (b and b' share an
    XCD exactly when b = b' mod 8; which XCD workgroup 0 gets depends on what was launched before)
    and that a CU holds two 4-wave workgroups of the 128x128 fp64 kernel (66 048 B of LDS each)."""
    torch = torch_mod()
    blocks = 1024
    out = torch.zeros(16 * blocks, dtype=torch.int32, device="cuda")
    assert xg.xgemm_hwid_probe(blocks, 66048, out) == 0
    torch.cuda.synchronize()
    rec = out.cpu().numpy().astype(np.uint32).reshape(blocks, 4, 4)
    assert np.array_equal(rec[:, 0, 2], np.arange(blocks))          # workgroup index as written
    xcc = rec[:, 0, 1] & 0xF
    assert np.array_equal(xcc, (np.arange(blocks) + int(xcc[0])) % 8)
    hw = rec[:512, 0, 0]
    cu_key = (xcc[:512].astype(np.int64) << 16) | (((hw >> 13) & 7) << 8) | (((hw >> 12) & 1) << 4) | ((hw >> 8) & 0xF)
    _, counts = np.unique(cu_key, return_counts=True)
    assert counts.size == 256 and np.all(counts == 2)


# --------------------------------------------------------------------------
# configuration 1: dgemm 256^3, alpha = 1, beta = 0, minimal ld
# --------------------------------------------------------------------------
def test_config1_dgemm_256():
    rng = si.rng_for(1)
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "N", 256, 256, 256)
    ratio = check_full(xg, "N", "N", 256, 256, 256, 1.0, A, lda, B, ldb, 0.0, C, ldc)
    print("config1 max err/bound", ratio, xg.xgemm_last_kernel_name())
    assert ratio < 1.0


# --------------------------------------------------------------------------
# every variant x every transpose pair x aligned / unaligned, ragged shapes
# --------------------------------------------------------------------------
def variant_cases():
    out = []
    for dtype, prec in ((np.float64, "d"), (np.float32, "s")):
        for v in range(16):
            out.append((dtype, prec, v))
    return out


@pytest.mark.parametrize("dtype,prec,variant", variant_cases())
def test_every_variant_ragged_shapes(dtype, prec, variant):
    if xg.xgemm_variant_name(prec, variant) is None:
        pytest.skip("no such variant")
    rng = si.rng_for(91, variant)
    # several tiles plus a ragged tail in every dimension; k tail not a multiple of the MFMA depth
    shapes = [(300, 275, 83), (129, 64, 16), (1, 1, 1), (17, 513, 5), (260, 3, 130)]
    for (m, n, k), ta, tb in itertools.product(shapes, TRANS, TRANS):
        for pad in ((0, 0, 0), (2, 4, 6) if dtype == np.float64 else (4, 8, 4), (1, 3, 5)):
            A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad, dtype)
            assert xg.xgemm_force_variant(variant) == 0
            ratio = check_full(xg, ta, tb, m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc)
            assert xg.xgemm_last_kernel_name() == xg.xgemm_variant_name(prec, variant)
            assert ratio < 1.0


@pytest.mark.parametrize("dtype,prec,variant", variant_cases())
def test_every_variant_integer_bit_exact(dtype, prec, variant):
    if xg.xgemm_variant_name(prec, variant) is None:
        pytest.skip("no such variant")
    rng = si.rng_for(92, variant)
    R = 1000 if dtype == np.float64 else 8
    for (m, n, k), (ta, tb) in zip([(256, 256, 256), (384, 200, 96), (131, 257, 67), (512, 128, 1024)],
                                    itertools.product(TRANS, TRANS)):
        for alpha, beta, pad in [(1.0, 0.0, (0, 0, 0)), (-1.0, 1.0, (0, 0, 0)), (2.0, -1.0, (1, 1, 1))]:
            A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad, dtype, "int", R)
            assert xg.xgemm_force_variant(variant) == 0
            out = run_real(xg, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc)
            want = C.copy()
            assert oracle.gemm_work(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, want, ldc) == 0
            assert np.array_equal(out, want, equal_nan=True)


def test_element_wise_fallback_kernels():
    """The fallback for leading dimensions beyond the 32-bit slab offsets cannot be
    reached with matrices that fit a test; a tuning switch read at load time sends
    unaligned operands there, so it is exercised in a child process."""
    import os
    import subprocess
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    env = dict(os.environ, XGEMM_REQUIRE_ALIGNED="1")
    r = subprocess.run([sys.executable, "-u", os.path.join(here, "fallback_case.py")], env=env, capture_output=True,
                       text=True, timeout=300)
    assert r.returncode == 0 and "fallback ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]


# --------------------------------------------------------------------------
# closed forms and scalar paths (automatic variant choice)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", DTYPES)
def test_ones_identity_and_scalar_paths(dtype):
    torch = torch_mod()
    m, n, k = 200, 150, 333
    # all ones: C == k exactly, NaN in C overwritten because beta == 0
    A, B = si.constant(m, k, m + 2, dtype), si.constant(k, n, k + 2, dtype)
    C = si.constant(m, n, m + 2, dtype, value=np.nan)
    out = run_real(xg, "N", "N", m, n, k, 1.0, A, m + 2, B, k + 2, 0.0, C, m + 2)
    assert np.array_equal(out[:, :m], np.full((n, m), k, dtype=dtype))
    assert np.all(np.isnan(out[:, m:]))
    # identity on the left: C = alpha X + beta C exactly
    rng = si.rng_for(93, 0)
    X, C0 = si.uniform(rng, m, n, m, dtype), si.uniform(rng, m, n, m, dtype)
    out = run_real(xg, "N", "N", m, n, m, 1.0, si.identity(m, dtype=dtype), m, X, m, 1.0, C0, m)
    assert np.array_equal(out, X + C0)
    # alpha == 0: A, B never read (NaN there, and also NULL)
    nanA, nanB = np.full((k, m), np.nan, dtype=dtype), np.full((n, k), np.nan, dtype=dtype)
    for beta in (0.0, -1.0, 2.0, 0.5):
        out = run_real(xg, "N", "N", m, n, k, 0.0, nanA, m, nanB, k, beta, C0, m)
        assert np.array_equal(out, (dtype(beta) * C0).astype(dtype))
        assert xg.xgemm_last_kernel_name() == "scale"
    out = run_real(xg, "N", "N", m, n, k, 0.0, None, m, None, k, 2.0, C0, m)
    assert np.array_equal(out, 2 * C0)
    # k == 0 behaves like alpha == 0; beta == 0 then stores zeros over NaN
    out = run_real(xg, "N", "N", m, n, 0, 1.0, None, m, None, 1, 0.0, np.full((n, m), np.nan, dtype=dtype), m)
    assert np.array_equal(out, np.zeros((n, m), dtype=dtype))
    # quick returns leave C untouched
    out = run_real(xg, "N", "N", m, n, k, 0.0, None, m, None, k, 1.0, C0, m)
    assert np.array_equal(out, C0) and xg.xgemm_last_kernel_name() == "none"
    out = run_real(xg, "N", "N", 0, n, k, 1.0, None, 1, None, k, 0.0, C0, m)
    assert np.array_equal(out, C0)
    # beta == 0 with NaN in C and a real product
    A, lda, B, ldb, _, ldc = make_operands(rng, "T", "T", m, n, k, (0, 0, 0), dtype)
    Cn = np.full((n, m), np.nan, dtype=dtype)
    out = run_real(xg, "T", "T", m, n, k, 1.0, A, lda, B, ldb, 0.0, Cn, m)
    assert np.all(np.isfinite(out))
    # illegal argument: nothing is written
    dC = to_dev(C0)
    f = xg.xgemm_dgemm if dtype == np.float64 else xg.xgemm_sgemm
    assert f("N", "N", m, n, k, 1.0, dC, m - 1, dC, k, 0.0, dC, m) == -8
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C0)


@pytest.mark.parametrize("dtype", DTYPES)
def test_run_to_run_determinism(dtype):
    rng = si.rng_for(94, 0)
    m, n, k = 640, 512, 700
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "N", m, n, k, (0, 0, 0), dtype)
    outs = [run_real(xg, "N", "N", m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc) for _ in range(3)]
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_non_default_stream():
    torch = torch_mod()
    rng = si.rng_for(94, 1)
    m, n, k = 256, 384, 128
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "T", m, n, k)
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    assert xg.xgemm_dgemm("N", "T", m, n, k, 1.0, dA, lda, dB, ldb, 1.0, dC, ldc, stream=s) == 0
    s.synchronize()
    want = C.copy()
    _, Cref, G = oracle.gemm_ext("N", "T", m, n, k, 1.0, A, lda, B, ldb, 1.0, C, ldc)
    assert oracle.bound_violations(dC.cpu().numpy(), Cref, G, k, oracle.U64)[0] == 0


# --------------------------------------------------------------------------
# configuration 2: dgemm squares with padded ld, alpha = 1.5, beta = -0.5
# --------------------------------------------------------------------------
@pytest.mark.parametrize("nsz", [512, 1024])
def test_config2_dgemm_square_full_check(nsz):
    rng = si.rng_for(2, nsz)
    ld = si.padded_ld(nsz)
    A, B, C = (si.uniform(rng, nsz, nsz, ld) for _ in range(3))
    ratio = check_full(xg, "N", "N", nsz, nsz, nsz, 1.5, A, ld, B, ld, -0.5, C, ld)
    print("config2", nsz, "max err/bound", ratio, xg.xgemm_last_kernel_name())


@pytest.mark.parametrize("nsz", [2048, 4096, 8192])
def test_config2_dgemm_square_large_full_check(nsz):
    """The sizes the benchmark times, in its launch configuration (padded leading dimensions,
    alpha 1.5, beta -0.5), every element against the extended-precision oracle."""
    rng = si.rng_for(2, nsz)
    ld = si.padded_ld(nsz)
    A, B, C = (si.uniform(rng, nsz, nsz, ld) for _ in range(3))
    out = run_real(xg, "N", "N", nsz, nsz, nsz, 1.5, A, ld, B, ld, -0.5, C, ld)
    kern = xg.xgemm_last_kernel_name()
    ratio = check_out_full(out, "N", "N", nsz, nsz, nsz, 1.5, A, ld, B, ld, -0.5, C, ld, label=f"config2 {nsz}")
    print("config2", nsz, "every element, max err/bound", ratio, kern)


def test_headline_size_integer_data_bit_exact():
    """8192^3 on integer-valued operands: every partial sum is exactly representable, so any
    summation order gives the same bits and the working-precision oracle is an exact reference
    for every element (numpy's float64 matmul on the same data is a third opinion)."""
    nsz = 8192
    rng = si.rng_for(2, 1)
    ld = si.padded_ld(nsz)
    A, B, C = (si.integers(rng, nsz, nsz, ld, R=1000) for _ in range(3))
    out = run_real(xg, "N", "N", nsz, nsz, nsz, 2.0, A, ld, B, ld, -1.0, C, ld)
    want = C.copy()
    assert oracle.gemm_work("N", "N", nsz, nsz, nsz, 2.0, A, ld, B, ld, -1.0, want, ld) == 0
    assert np.abs(want[:, :nsz]).max() < 2.0 ** 53
    assert np.array_equal(out, want, equal_nan=True)
    # column-major product C = A B is, on the (cols, ld) arrays, out_rows = B_rows @ A_rows
    assert np.array_equal(out[:, :nsz], 2.0 * (B[:, :nsz] @ A[:, :nsz]) - C[:, :nsz])
    # all ones at the same size: C == k
    ones = si.constant(nsz, nsz, ld)
    out = run_real(xg, "N", "N", nsz, nsz, nsz, 1.0, ones, ld, ones, ld, 0.0, C, ld)
    assert np.array_equal(out[:, :nsz], np.full((nsz, nsz), float(nsz)))


# --------------------------------------------------------------------------
# configuration 3: sgemm squares (alpha = beta = 1, minimal ld) and transposes at 4096
# --------------------------------------------------------------------------
def test_config3_sgemm_1024_full_check():
    rng = si.rng_for(3, 1024)
    nsz = 1024
    A, B, C = (si.uniform(rng, nsz, nsz, nsz, np.float32) for _ in range(3))
    ratio = check_full(xg, "N", "N", nsz, nsz, nsz, 1.0, A, nsz, B, nsz, 1.0, C, nsz)
    print("config3 1024 max err/bound", ratio, xg.xgemm_last_kernel_name())


@pytest.mark.parametrize("nsz,ta,tb", [(4096, "N", "N"), (4096, "N", "T"), (4096, "T", "N"), (4096, "T", "T"),
                                       (8192, "N", "N")])
def test_config3_sgemm_large_full_check(nsz, ta, tb):
    """Every element against the oracle that accumulates in double."""
    rng = si.rng_for(3, nsz + (ta == "T") + 2 * (tb == "T"))
    A, B, C = (si.uniform(rng, nsz, nsz, nsz, np.float32) for _ in range(3))
    out = run_real(xg, ta, tb, nsz, nsz, nsz, 1.0, A, nsz, B, nsz, 1.0, C, nsz)
    kern = xg.xgemm_last_kernel_name()
    ratio = check_out_full(out, ta, tb, nsz, nsz, nsz, 1.0, A, nsz, B, nsz, 1.0, C, nsz, chunk=2048,
                           label=f"config3 {nsz} {ta}{tb}")
    print("config3", nsz, ta + tb, "every element, max err/bound", ratio, kern)


def test_config3_sgemm_16384_sampled():
    """The one size whose full oracle (8.8 Tflop) does not fit a test: 64 full rows, 64 full
    columns and 2^16 random entries."""
    nsz = 16384
    rng = si.rng_for(3, nsz)
    A, B, C = (si.uniform(rng, nsz, nsz, nsz, np.float32) for _ in range(3))
    out = run_real(xg, "N", "N", nsz, nsz, nsz, 1.0, A, nsz, B, nsz, 1.0, C, nsz)
    assert np.all(np.isfinite(out))
    I, J = si.sample_indices(rng, nsz, nsz, 64, 64, 65536)
    ratio = check_samples(out, "N", "N", nsz, nsz, nsz, 1.0, A, nsz, B, nsz, 1.0, C, nsz, I, J)
    print("config3", nsz, "sampled max err/bound", ratio, xg.xgemm_last_kernel_name())


# --------------------------------------------------------------------------
# configuration 4: rank-k updates (alpha = -1, beta = 1, normal entries), ragged edges
# --------------------------------------------------------------------------
@pytest.mark.parametrize("mn,k", [(4096, 64), (4096, 128), (4096, 256), (16384, 64), (16384, 128), (16384, 256)])
def test_config4_rank_k_update(mn, k):
    """Rank-k updates, every element (the depth is small, so the full oracle is cheap)."""
    rng = si.rng_for(4, mn + k)
    A, B, C = si.normal(rng, mn, k), si.normal(rng, k, mn), si.normal(rng, mn, mn)
    out = run_real(xg, "N", "N", mn, mn, k, -1.0, A, mn, B, k, 1.0, C, mn)
    kern = xg.xgemm_last_kernel_name()
    ratio = check_out_full(out, "N", "N", mn, mn, k, -1.0, A, mn, B, k, 1.0, C, mn, chunk=2048,
                           label=f"config4 {mn} k={k}")
    print("config4", mn, k, "every element, max err/bound", ratio, kern)


@pytest.mark.parametrize("pads", [(0, 0, 0), (7, 7, 7)])
def test_config4_ragged_4097_3001_257(pads):
    m, n, k = 4097, 3001, 257
    rng = si.rng_for(4, 1)
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "N", m, n, k, pads, np.float64, "normal")
    ratio = check_full(xg, "N", "N", m, n, k, -1.0, A, lda, B, ldb, 1.0, C, ldc)
    print("config4 ragged", pads, "max err/bound", ratio, xg.xgemm_last_kernel_name())


# --------------------------------------------------------------------------
# configuration 5: complex GEMM on split planes
# --------------------------------------------------------------------------
def zoperands(rng, ta, tb, m, n, k, kind="uniform", pad=(0, 0, 0)):
    ra, ca = si.operand_shape(ta, m, k)
    rb, cb = si.operand_shape(tb, k, n)
    lda, ldb, ldc = ra + pad[0], rb + pad[1], m + pad[2]
    if kind == "int":
        gen = lambda r, c, ld: si.integers(rng, r, c, ld, R=100)
    else:
        gen = lambda r, c, ld: si.uniform(rng, r, c, ld)
    return [gen(ra, ca, lda), gen(ra, ca, lda), gen(rb, cb, ldb), gen(rb, cb, ldb),
            gen(m, n, ldc), gen(m, n, ldc)], lda, ldb, ldc


def run_z(ta, tb, m, n, k, alpha, planes, lda, ldb, beta, ldc):
    torch = torch_mod()
    d = [to_dev(P) for P in planes]
    lw = xg.xgemm_zgemm_worksize(m, n, alpha, beta)
    work = torch.full((max(lw, 1),), float("nan"), dtype=torch.float64, device="cuda")
    rc = xg.xgemm_zgemm_split(ta, tb, m, n, k, alpha, d[0], d[1], lda, d[2], d[3], ldb, beta, d[4], d[5], ldc,
                              work if lw else None, lw)
    torch.cuda.synchronize()
    assert rc == 0
    return d[4].cpu().numpy(), d[5].cpu().numpy()


@pytest.mark.parametrize("ta,tb", list(itertools.product("NTC", "NTC")))
def test_zgemm_small_full_check(ta, tb):
    rng = si.rng_for(5, 100)
    m, n, k = 150, 131, 77
    for alpha, beta in [((1.0, 0.0), (0.0, 0.0)), ((1.5, 0.0), (-0.5, 0.0)), ((0.75, -1.25), (0.5, 2.0)),
                        ((0.0, 1.0), (0.0, 0.0))]:
        planes, lda, ldb, ldc = zoperands(rng, ta, tb, m, n, k, pad=(2, 4, 6))
        if beta == (0.0, 0.0):
            planes[4][:, :m] = np.nan
            planes[5][:, :m] = np.nan
        Or, Oi = run_z(ta, tb, m, n, k, alpha, planes, lda, ldb, beta, ldc)
        info, Rr, Ri, Gr, Gi = oracle.zgemm_split_ext(ta, tb, m, n, k, alpha, *planes[:2], lda, *planes[2:4], ldb,
                                                      beta, *planes[4:], ldc)
        assert info == 0
        for O, R, G, P in ((Or, Rr, Gr, planes[4]), (Oi, Ri, Gi, planes[5])):
            nviol, ratio = oracle.bound_violations(O[:, :m], R, G, k, oracle.U64, factor=8.0)
            assert nviol == 0, (ta, tb, alpha, beta, ratio)
            assert np.array_equal(O[:, m:], P[:, m:], equal_nan=True)


def test_zgemm_gaussian_integers_bit_exact():
    rng = si.rng_for(5, 101)
    m, n, k = 200, 260, 129
    for (ta, tb), (alpha, beta) in zip([("N", "N"), ("C", "T"), ("T", "C")],
                                       [((1.0, 0.0), (0.0, 0.0)), ((2.0, 0.0), (-1.0, 0.0)), ((2.0, -1.0), (1.0, 3.0))]):
        planes, lda, ldb, ldc = zoperands(rng, ta, tb, m, n, k, kind="int", pad=(0, 2, 0))
        Or, Oi = run_z(ta, tb, m, n, k, alpha, planes, lda, ldb, beta, ldc)
        Wr, Wi = planes[4].copy(), planes[5].copy()
        assert oracle.zgemm_split_work(ta, tb, m, n, k, alpha, *planes[:2], lda, *planes[2:4], ldb, beta, Wr, Wi, ldc) == 0
        assert np.array_equal(Or, Wr, equal_nan=True) and np.array_equal(Oi, Wi, equal_nan=True)


def test_config5_zgemm_4096_sampled():
    nsz = 4096
    rng = si.rng_for(5, nsz)
    planes, lda, ldb, ldc = zoperands(rng, "N", "N", nsz, nsz, nsz)
    alpha, beta = (1.0, 0.0), (0.0, 0.0)
    Or, Oi = run_z("N", "N", nsz, nsz, nsz, alpha, planes, lda, ldb, beta, ldc)
    I, J = si.sample_indices(rng, nsz, nsz, 2, 2, 4096)
    info, rr, ri, gr, gi = oracle.zgemm_split_samples("N", "N", nsz, nsz, nsz, alpha, *planes[:2], lda,
                                                      *planes[2:4], ldb, beta, *planes[4:], ldc, I, J)
    assert info == 0
    for O, r, g in ((Or, rr, gr), (Oi, ri, gi)):
        nviol, ratio = oracle.bound_violations(O[J, I], r, g, nsz, oracle.U64, factor=8.0)
        assert nviol == 0, ratio
        print("config5 zgemm 4096 sampled max err/bound", ratio)


def test_latency_probe_reports_plausible_chains():
    """The probe behind the measured latency table: every chain takes a positive time, a dependent
    FP64 multiply-add costs a few cycles, and the slower kinds are slower (matrix instruction,
    LDS round trip, lane read) -- the ordering the block kernels were designed around."""
    torch = torch_mod()
    out = torch.zeros(8, dtype=torch.int64, device="cuda")
    sink = torch.zeros(64, dtype=torch.float64, device="cuda")
    iters = 2000
    for _ in range(2):
        assert xg.xgemm_latency_probe(out, sink, iters) == 0
        torch.cuda.synchronize()
    t = out.cpu().numpy().astype(np.float64)
    per = np.array([8, 8, 8, 4, 4, 4, 8, 4], dtype=np.float64)
    ns = 10.0 * t / (iters * per)
    assert np.all(ns > 0.5) and np.all(ns < 500.0), ns
    fma64, fma32, rsq, lds, mfma64, mfma_valu, lane, mfma32 = ns
    assert fma64 < 20.0 and fma32 < 20.0
    assert mfma64 > 2 * fma64 and lds > 2 * fma64 and lane > fma64 and rsq > fma64
    assert xg.xgemm_latency_probe(out, sink, 0) != 0
