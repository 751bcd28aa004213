"""GPU parity of the workspace routines (tail tiles split along K): same bound as
the plain routines, bit-exact on integer data, independent of arrival order, and
the workspace counters left zero."""
import itertools

import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import make_operands, make_syrk_operands, to_dev, torch_mod, unit_roundoff

pytestmark = pytest.mark.gpu

CNT_BYTES = 8192
SPLIT_VARIANTS = [(np.float64, "d", 0), (np.float32, "s", 0), (np.float32, "s", 1)]


@pytest.fixture(autouse=True)
def _auto():
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)
    yield
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)


@pytest.fixture(scope="module")
def ws():
    torch = torch_mod()
    nbytes = xg.xgemm_workspace_bytes()
    w = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    w.fill_(0xA5)                     # stale contents must not matter beyond the counters
    assert xg.xgemm_workspace_init(w, nbytes) == 0
    torch.cuda.synchronize()
    return w, nbytes


def counters_are_zero(w):
    return not bool(w[:CNT_BYTES].any().item())


def run_ws(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, w, lw):
    torch = torch_mod()
    f = xg.xgemm_dgemm_ws if C.dtype == np.float64 else xg.xgemm_sgemm_ws
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    assert f(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc, w, lw) == 0
    torch.cuda.synchronize()
    return dC.cpu().numpy()


@pytest.mark.parametrize("dtype,prec,variant", SPLIT_VARIANTS)
def test_forced_split_counts_ragged_shapes(ws, dtype, prec, variant):
    w, lw = ws
    rng = si.rng_for(101, variant)
    # all tiles are tail tiles here (fewer tiles than slots); K tails of every kind
    for (m, n, k), pieces, (ta, tb) in zip(
            [(300, 275, 331), (129, 64, 1024), (515, 260, 200), (1, 1, 64), (260, 300, 130), (700, 130, 517)],
            [2, 16, 3, 4, 2, 5], itertools.cycle(itertools.product("NT", "NT"))):
        for pad in ((0, 0, 0), (1, 3, 5)):
            A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad, dtype)
            assert xg.xgemm_force_variant(variant) == 0 and xg.xgemm_force_split(pieces) == 0
            out = run_ws(ta, tb, m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc, w, lw)
            nslab = -(-k // 16)
            assert xg.xgemm_last_split() == max(1, min(pieces, nslab // 4)), (m, n, k, pieces)
            info, Cref, G = oracle.gemm_ext(ta, tb, m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc)
            nviol, ratio = oracle.bound_violations(out[:, :m], Cref, G, k, unit_roundoff(dtype), 4.0)
            assert info == 0 and nviol == 0, (m, n, k, pieces, nviol, ratio)
            assert np.array_equal(out[:, m:], C[:, m:], equal_nan=True)
            assert counters_are_zero(w)


@pytest.mark.parametrize("dtype,prec,variant", SPLIT_VARIANTS)
def test_split_integer_bit_exact_and_repeatable(ws, dtype, prec, variant):
    w, lw = ws
    rng = si.rng_for(102, variant)
    R = 1000 if dtype == np.float64 else 8
    m, n, k = 384, 520, 2048
    A, lda, B, ldb, C, ldc = make_operands(rng, "T", "N", m, n, k, (1, 1, 1), dtype, "int", R)
    want = C.copy()
    assert oracle.gemm_work("T", "N", m, n, k, 2.0, A, lda, B, ldb, -1.0, want, ldc) == 0
    xg.xgemm_force_variant(variant)
    for pieces in (0, 2, 7, 32):
        xg.xgemm_force_split(pieces)
        out = run_ws("T", "N", m, n, k, 2.0, A, lda, B, ldb, -1.0, C, ldc, w, lw)
        assert xg.xgemm_last_split() == max(pieces, 1)
        assert np.array_equal(out, want, equal_nan=True)
    # floating-point data: the pieces are added in a fixed order, so repeated runs agree bit for bit
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "T", m, n, k, (0, 0, 0), dtype)
    xg.xgemm_force_split(8)
    first = run_ws("N", "T", m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc, w, lw)
    for _ in range(3):
        assert np.array_equal(first, run_ws("N", "T", m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc, w, lw), equal_nan=True)
    assert counters_are_zero(w)


def test_model_splits_only_the_last_round_and_small_workspaces_split_less(ws):
    w, lw = ws
    torch = torch_mod()
    rng = si.rng_for(103, 0)
    # 26 x 20 = 520 tiles of 128 x 128 on 512 slots: 512 whole tiles and 8 tail tiles
    m, n, k = 26 * 128, 20 * 128, 2048
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "N", m, n, k, (8, 8, 8), np.float64)
    dA, dB = to_dev(A), to_dev(B)
    I, J = si.sample_indices(rng, m, n, 4, 4, 4096)
    info, cref, gb = oracle.gemm_samples("N", "N", m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc, I, J)
    assert info == 0
    xg.xgemm_force_variant(0)     # the variant the tile count above is for; the split count stays the model's
    seen = []
    for nbytes in (lw, CNT_BYTES + 8 * 3 * 128 * 128 * 8, CNT_BYTES + 8 * 128 * 128 * 8, CNT_BYTES):
        dC = to_dev(C)
        assert xg.xgemm_dgemm_ws("N", "N", m, n, k, 1.5, dA, lda, dB, ldb, -0.5, dC, ldc, w, nbytes) == 0
        torch.cuda.synchronize()
        assert xg.xgemm_last_kernel_name() == "d_128x128x16_w2x2"
        seen.append(xg.xgemm_last_split())
        out = dC.cpu().numpy()
        nviol, ratio = oracle.bound_violations(out[J, I], cref, gb, k, oracle.U64, 4.0)
        assert nviol == 0, (nbytes, nviol, ratio)
    # room for 3 pieces per tile: a 3-way split, unless the model rates running the tail as quarter
    # tiles (which needs no workspace) cheaper than so shallow a split
    assert seen[0] >= 8 and seen[1] in (1, 3) and seen[2] == 1 and seen[3] == 1, seen
    assert counters_are_zero(w)
    # without a workspace the routine is the plain one
    dC = to_dev(C)
    assert xg.xgemm_dgemm_ws("N", "N", m, n, k, 1.5, dA, lda, dB, ldb, -0.5, dC, ldc, None, 0) == 0
    assert xg.xgemm_last_split() == 1
    assert xg.xgemm_dgemm_ws("N", "N", m, n, k, 1.5, dA, lda, dB, ldb, -0.5, dC, ldc, w.data_ptr() + 8, lw - 8) == -14
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_syrk_with_workspace(ws, dtype):
    w, lw = ws
    torch = torch_mod()
    rng = si.rng_for(104, 0)
    f = xg.xgemm_dsyrk_ws if dtype == np.float64 else xg.xgemm_ssyrk_ws
    xg.xgemm_force_variant(0)
    for (n, k), pieces, (uplo, trans) in zip([(515, 300), (300, 2048), (1000, 130)], [2, 16, 3],
                                              itertools.cycle(itertools.product("LU", "NT"))):
        A, lda, C, ldc = make_syrk_operands(rng, trans, n, k, (3, 5), dtype)
        xg.xgemm_force_split(pieces)
        dA, dC = to_dev(A), to_dev(C)
        assert f(uplo, trans, n, k, 1.5, dA, lda, -0.5, dC, ldc, w, lw) == 0
        torch.cuda.synchronize()
        assert xg.xgemm_last_split() > 1
        out = dC.cpu().numpy()
        info, Cref, G = oracle.syrk_ext(uplo, trans, n, k, 1.5, A, lda, -0.5, C, ldc)
        mask = oracle.triangle_mask(uplo, n)
        got = np.where(mask, out[:, :n], 0).astype(dtype)
        nviol, ratio = oracle.bound_violations(got, Cref, G, k, unit_roundoff(dtype), 4.0)
        assert info == 0 and nviol == 0, (n, k, pieces, nviol, ratio)
        keep = np.ones(C.shape, dtype=bool)
        keep[:, :n] = ~mask
        assert np.array_equal(out[keep], C[keep], equal_nan=True)
        assert counters_are_zero(w)
