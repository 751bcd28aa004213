"""GPU parity of the LU driver against the CPU oracle.  Several factorisations are correct when candidates
for a pivot tie or differ by a rounding, so the statement checked everywhere is the complete validity
statement (legal interchanges, no multiplier above one, |P A - L U| <= 4 min(m,n) u |L||U| element by element,
evaluated by the oracle in extended precision); equality with the oracle's interchanges and factors is asked
for where it is determined: matrices whose factorisation is exact, and tie-free random matrices."""
import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import to_dev, torch_mod, unit_roundoff
from lu_util import check_valid, perm_of, planted_lu, unpack

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto():
    xg.xgemm_tuning_reset()
    yield
    xg.xgemm_tuning_reset()


def run_getrf(m, n, A, lda, stream=None, ws=False):
    """ws False: xgemm_*getrf held to the leaves of one workgroup each (the route of a captured call);
    ws True: through xgemm_*getrf_ws with an exchange buffer full of ones (it needs no preparation), so that
    the panels are shared by all the workgroups their rows need; ws "auto": xgemm_*getrf as it comes (shared
    panels through the library's own exchange buffer)."""
    torch = torch_mod()
    dA = to_dev(A)
    k = max(min(m, n), 1)
    dpiv = torch.full((k,), -7, dtype=torch.int32, device="cuda")
    dinfo = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    if ws is True:
        f = xg.xgemm_dgetrf_ws if A.dtype == np.float64 else xg.xgemm_sgetrf_ws
        lwork = xg.xgemm_getrf_workspace_bytes()
        work = torch.full((lwork,), 0xFF, dtype=torch.uint8, device="cuda")
        assert f(m, n, dA, lda, dpiv, dinfo, work, lwork, stream=stream) == 0
    else:
        assert xg.xgemm_force_getrf_shared(-1 if ws == "auto" else 0) == 0
        f = xg.xgemm_dgetrf if A.dtype == np.float64 else xg.xgemm_sgetrf
        assert f(m, n, dA, lda, dpiv, dinfo, stream=stream) == 0
        assert xg.xgemm_force_getrf_shared(-1) == 0
    torch.cuda.synchronize()
    return dA.cpu().numpy(), dpiv.cpu().numpy()[:min(m, n)], int(dinfo.item())


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("panel,ws", [(-1, False), (16, False), (40, False), (-1, True), (16, True), (40, True), (-1, "auto"), (40, "auto")])
def test_planted_factorisations_are_recovered_exactly(dtype, panel, ws):
    """Every operation on these matrices is exact, so interchanges and factors must come out bit for bit,
    whatever the blocking: one leaf, several leaves, several panels, ragged last leaf and panel, tall, wide."""
    rng = si.rng_for(310, panel + 1)
    for m, n in [(1, 1), (7, 5), (5, 7), (8, 8), (9, 9), (64, 64), (200, 131), (131, 200), (300, 300), (517, 517), (1100, 700)]:
        A, L, U, perm = planted_lu(rng, m, n, dtype, ld=m + 3)
        assert xg.xgemm_force_getrf_panel(panel) == 0
        F, ipiv, info = run_getrf(m, n, A, m + 3, ws=ws)
        assert info == 0, (m, n)
        k = min(m, n)
        assert np.all(ipiv >= np.arange(1, k + 1)) and np.all(ipiv <= m)
        src, where = perm_of(ipiv, m), np.argsort(perm)
        assert np.array_equal(src[:k], perm[:k]), (m, n, panel)
        Lg, Ug = unpack(F, m, n)
        assert np.array_equal(Ug, U) and np.array_equal(Lg, L[where[src], :]), (m, n, panel)
        assert np.all(np.isnan(F[:, m:])), "padding rows were written"


@pytest.mark.parametrize("ws", [False, True, "auto"])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_random_matrices_every_element_and_against_the_oracle(dtype, ws):
    rng = si.rng_for(311, 0)
    u = unit_roundoff(dtype)
    for (m, n), panel in [((50, 50), -1), ((257, 257), 64), ((300, 120), -1), ((120, 300), 32), ((1000, 1000), -1),
                          ((777, 1031), 128), ((1031, 777), 24)]:
        A = si.uniform(rng, m, n, m + 1, dtype)
        assert xg.xgemm_force_getrf_panel(panel) == 0
        F, ipiv, info = run_getrf(m, n, A, m + 1, ws=ws)
        assert info == 0
        ratio = check_valid(m, n, A, m + 1, F, m + 1, ipiv, u)
        assert np.all(np.isnan(F[:, m:]))
        # tie-free data: the oracle makes the same choices, and the factors agree to rounding
        W = A.copy()
        oinfo, opiv = oracle.getrf(m, n, W, m + 1)
        assert oinfo == 0 and np.array_equal(ipiv, opiv), (m, n)
        tol = 64 * min(m, n) * u
        assert np.allclose(F[:, :m], W[:, :m], rtol=tol, atol=tol), (m, n)
        print("getrf", dtype.__name__, m, n, "panel", panel, "ws", ws, "max err/bound", ratio)


@pytest.mark.parametrize("ws", [False, True, "auto"])
def test_tie_rule_and_zero_pivots(ws):
    def run_getrf(*a):
        return globals()["run_getrf"](*a, ws=ws)
    # the first of equal candidates is taken (exact small integers: the arithmetic decides nothing)
    A = np.array([[2.0, -2.0, 2.0], [1.0, 3.0, 5.0], [0.0, 1.0, 4.0]])
    F, ipiv, info = run_getrf(3, 3, A, 3)
    W = A.copy()
    oinfo, opiv = oracle.getrf(3, 3, W, 3)
    assert info == 0 and list(ipiv) == [1, 2, 3] and np.array_equal(ipiv, opiv) and np.array_equal(F, W)
    # a matrix full of ties (entries -1, 0, 1): whatever is chosen, the statement must hold
    rng = si.rng_for(312, 0)
    n = 200
    A = si.integers(rng, n, n, n, np.float64, R=1)
    F, ipiv, info = run_getrf(n, n, A, n)
    if info == 0:
        check_valid(n, n, A, n, F, n, ipiv, oracle.U64)
    # zero columns: reported (first one), nothing divided, the elimination goes on
    Z = np.zeros((3, 4))
    F, ipiv, info = run_getrf(4, 3, Z, 4)
    assert info == 1 and list(ipiv) == [1, 2, 3] and not F.any()
    A = si.uniform(rng, 40, 40, 40)
    A[17, :] = 0.0                                           # column 18 is zero
    A[:, :] = A                                              # (col, row) layout: A[17] is the column
    F, ipiv, info = run_getrf(40, 40, A, 40)
    W = A.copy()
    oinfo, opiv = oracle.getrf(40, 40, W, 40)
    assert info == oinfo == 18 and np.array_equal(ipiv, opiv)
    assert np.allclose(F, W, rtol=1e-12, atol=1e-13)
    check_valid(40, 40, A, 40, F, 40, ipiv, oracle.U64)
    # ties across the stripes of a shared panel: the first row of the largest magnitude wins wherever it lies
    n = 700
    A = si.integers(rng, n, n, n, np.float64, R=1)
    A[0, :] = 0.0                                            # column 1: +-3 in rows 650, 300 and 129 only
    A[0, 650], A[0, 300], A[0, 129] = 3.0, -3.0, 3.0
    F, ipiv, info = run_getrf(n, n, A, n)
    assert ipiv[0] == 130
    if info == 0:
        check_valid(n, n, A, n, F, n, ipiv, oracle.U64)


@pytest.mark.parametrize("ws", [False, True, "auto"])
@pytest.mark.parametrize("dtype,n", [(np.float64, 4096), (np.float64, 8192), (np.float32, 8192)])
def test_full_size_sampled(dtype, n, ws):
    """The sizes of the sweep: legal interchanges, multipliers within one, the residual bound on 16 full rows,
    16 full columns and 2^15 entries; the planted matrix of the same size bit for bit."""
    rng = si.rng_for(313, n)
    A = si.uniform(rng, n, n, n, dtype)
    F, ipiv, info = run_getrf(n, n, A, n, ws=ws)
    assert info == 0
    I, J = si.sample_indices(rng, n, n, 16, 16, 1 << 15)
    ratio = check_valid(n, n, A, n, F, n, ipiv, unit_roundoff(dtype), I=I, J=J)
    print("getrf", dtype.__name__, n, "sampled max err/bound", ratio)
    if dtype == np.float64 and n == 4096:
        A, L, U, perm = planted_lu(rng, n, n, dtype)
        F, ipiv, info = run_getrf(n, n, A, n, ws=ws)
        Lg, Ug = unpack(F, n, n)
        assert info == 0 and np.array_equal(perm_of(ipiv, n), perm) and np.array_equal(Ug, U) and np.array_equal(Lg, L)


def test_on_a_stream_of_the_callers_and_twice_the_same_bits():
    torch = torch_mod()
    rng = si.rng_for(314, 0)
    n = 900
    A = si.uniform(rng, n, n, n)
    side = torch.cuda.Stream()
    for ws in (False, "auto"):
        F1, p1, i1 = run_getrf(n, n, A, n, ws=ws)
        F2, p2, i2 = run_getrf(n, n, A, n, stream=side, ws=ws)
        assert i1 == 0 and i2 == 0 and np.array_equal(p1, p2) and np.array_equal(F1, F2)


def test_shared_panels_agree_with_the_leaves_and_repeat_bit_for_bit():
    """Tie-free data: both routes take the same pivots; the shared panels give the same bits twice in a row
    (nothing in them depends on which workgroup arrives first)."""
    rng = si.rng_for(315, 0)
    for m, n in [(1500, 1500), (2300, 900), (900, 2300)]:
        A = si.uniform(rng, m, n, m)
        F0, p0, i0 = run_getrf(m, n, A, m)
        F1, p1, i1 = run_getrf(m, n, A, m, ws=True)
        F2, p2, i2 = run_getrf(m, n, A, m, ws=True)
        assert i0 == i1 == i2 == 0 and np.array_equal(p0, p1) and np.array_equal(p1, p2)
        assert np.array_equal(F1, F2)
        tol = 64 * min(m, n) * oracle.U64 * np.abs(F0[:, :m]).max()       # entries of U grow beyond one
        assert np.allclose(F0, F1, rtol=0.0, atol=tol)


def test_a_wait_that_times_out_ends_the_call_with_info_minus_one():
    """With no polls allowed a workgroup of a shared panel gives up unless all others had arrived already; the
    others follow, every kernel ends, *info is -1, and the next call with the default limit is right again."""
    torch = torch_mod()
    rng = si.rng_for(316, 0)
    n = 2048
    A = si.uniform(rng, n, n, n)
    assert xg.xgemm_force_getrf_spin_limit(0) == 0
    F, ipiv, info = run_getrf(n, n, A, n, ws=True)
    assert info in (0, -1)
    if info == 0:
        check_valid(n, n, A, n, F, n, ipiv, oracle.U64)
    xg.xgemm_tuning_reset()
    F, ipiv, info = run_getrf(n, n, A, n, ws=True)
    assert info == 0
    I, J = si.sample_indices(rng, n, n, 8, 8, 1 << 12)
    check_valid(n, n, A, n, F, n, ipiv, oracle.U64, I=I, J=J)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_tall_panels_up_to_one_workgroup_per_compute_unit_and_beyond(dtype):
    """Shared panels of 157, 256 (every compute unit of the device holds a stripe) and 258 stripes (more than
    the device has compute units: that panel goes the way of the leaves, the later ones are shared again):
    in fp64 the same interchanges as the oracle and the factors to rounding; the validity statement on sampled
    rows and columns."""
    u = unit_roundoff(dtype)
    for m, n in [(20000, 200), (32768, 130), (33000, 260)]:
        rng = si.rng_for(317, m)
        A = si.uniform(rng, m, n, m, dtype)
        F, ipiv, info = run_getrf(m, n, A, m, ws=True)
        assert info == 0
        if dtype == np.float64:       # (in fp32 the two largest of 33000 entries are within a rounding often enough)
            W = A.copy()
            oinfo, opiv = oracle.getrf(m, n, W, m)
            assert oinfo == 0 and np.array_equal(ipiv, opiv), (m, n)
            tol = 64 * n * u * max(1.0, float(np.abs(W).max()))
            assert np.allclose(F, W, rtol=0.0, atol=tol), (m, n)
        I, J = si.sample_indices(rng, m, n, 8, 8, 1 << 12)
        check_valid(m, n, A, m, F, m, ipiv, u, I=I, J=J)


def test_factorisations_on_two_streams_at_once_are_ordered_by_the_library():
    """Two factorisations with shared panels enqueued back to back on two streams, each with panels of 40 or
    more workgroups, and a third through the caller's own buffer: the library orders them on the device (their
    workgroups wait for each other, so they must not compete for compute units), and all three give the bits
    of a factorisation that ran alone."""
    torch = torch_mod()
    rng = si.rng_for(318, 0)
    n = 5200
    A = si.uniform(rng, n, n, n)
    want, wpiv, winfo = run_getrf(n, n, A, n, ws="auto")
    assert winfo == 0
    streams = [torch.cuda.Stream() for _ in range(3)]
    dAs = [to_dev(A) for _ in range(3)]
    pivs = [torch.zeros(n, dtype=torch.int32, device="cuda") for _ in range(3)]
    infos = [torch.full((1,), -7, dtype=torch.int32, device="cuda") for _ in range(3)]
    lw = xg.xgemm_getrf_workspace_bytes()
    work = torch.empty(lw, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    assert xg.xgemm_dgetrf(n, n, dAs[0], n, pivs[0], infos[0], stream=streams[0]) == 0
    assert xg.xgemm_dgetrf(n, n, dAs[1], n, pivs[1], infos[1], stream=streams[1]) == 0
    assert xg.xgemm_dgetrf_ws(n, n, dAs[2], n, pivs[2], infos[2], work, lw, stream=streams[2]) == 0
    torch.cuda.synchronize()
    for k in range(3):
        assert int(infos[k].item()) == 0
        assert np.array_equal(pivs[k].cpu().numpy(), wpiv) and np.array_equal(dAs[k].cpu().numpy(), want), k


def test_many_random_shapes_give_the_same_bits_on_every_run_and_through_either_buffer():
    """The pivot of a column is agreed between workgroups that run at their own pace; nothing in the result may
    depend on who arrives when.  Forty random shapes, both precisions: the library's buffer, a caller's buffer and
    the library's again give the same factors and interchanges bit for bit."""
    torch = torch_mod()
    lw = xg.xgemm_getrf_workspace_bytes()
    work = torch.empty(lw, dtype=torch.uint8, device="cuda")
    shapes = np.random.default_rng(12345)
    for it in range(40):
        m, n = int(shapes.integers(200, 7000)), int(shapes.integers(200, 2500))
        dtype = np.float64 if it % 3 else np.float32
        A = si.uniform(si.rng_for(319, it), m, n, m, dtype)
        outs = [run_getrf(m, n, A, m, ws=ws) for ws in ("auto", True, "auto")]
        assert all(o[2] == 0 for o in outs), (it, m, n)
        for o in outs[1:]:
            assert np.array_equal(outs[0][0], o[0]) and np.array_equal(outs[0][1], o[1]), (it, m, n)
