"""The entry point for callers that cannot allocate (xgemm_dgemm_static): through the C ABI, against
xgemm_dgemm_ws given a full-size workspace (the same plan, so the same bits) and against the oracle's
bound, on calls in a row that share the device's static scratch, the later ones with smaller inputs."""
import numpy as np
import pytest

import oracle
import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import make_operands, to_dev, torch_mod

pytestmark = pytest.mark.gpu


def _both(ta, tb, m, n, k, alpha, beta, rng, pad=(0, 0, 0)):
    """Run the static entry point and the workspace one on the same operands; return what is needed to compare."""
    torch = torch_mod()
    A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, pad)
    dA, dB = to_dev(A), to_dev(B)
    d1, d2 = to_dev(C), to_dev(C)
    lw = xg.xgemm_workspace_bytes()
    work = torch.zeros(lw, dtype=torch.uint8, device="cuda")
    assert xg.xgemm_workspace_init(work, lw) == 0
    rc_ws = xg.xgemm_dgemm_ws(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, d2, ldc, work, lw)
    split_ws, kern_ws = xg.xgemm_last_split(), xg.xgemm_last_kernel_name()
    rc_st = xg.xgemm_dgemm_static(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, d1, ldc)
    split_st, kern_st = xg.xgemm_last_split(), xg.xgemm_last_kernel_name()
    torch.cuda.synchronize()
    return dict(A=A, lda=lda, B=B, ldb=ldb, C=C, ldc=ldc, rc_ws=rc_ws, rc_st=rc_st, out_ws=d2.cpu().numpy(),
                out_st=d1.cpu().numpy(), split_ws=split_ws, split_st=split_st, kern_ws=kern_ws, kern_st=kern_st)


def test_static_scratch_entry_matches_workspace_entry_on_calls_in_a_row():
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)
    rng = si.rng_for(97, 0)
    # (shape, expected to split): 3072 x 3072 x 1000 uses the whole array (4 pieces x 64 tail tiles x 128 KiB; at
    # this depth the tail cannot go to quarter tiles instead), the next calls are smaller and find the previous
    # call's partial sums and counters in the array
    cases = [(("N", "N", 3072, 3072, 1000), True), (("N", "T", 768, 768, 2048), True),
             (("T", "N", 3328, 2560, 2048), True), (("N", "N", 515, 259, 4100), True),
             (("N", "N", 1024, 1024, 512), False), (("T", "T", 300, 275, 83), False)]
    for (ta, tb, m, n, k), splits in cases:
        print("static entry", ta, tb, m, n, k, flush=True)
        r = _both(ta, tb, m, n, k, 1.5, -0.5, rng, pad=(0, 0, 0) if m % 8 == 0 else (1, 3, 5))
        assert r["rc_ws"] == 0 and r["rc_st"] == 0, (r["rc_ws"], r["rc_st"])
        assert (r["split_st"] > 1) == splits and r["split_st"] == r["split_ws"] and r["kern_st"] == r["kern_ws"]
        assert np.array_equal(r["out_st"], r["out_ws"], equal_nan=True)
        info, Cref, G = oracle.gemm_ext(ta, tb, m, n, k, 1.5, r["A"], r["lda"], r["B"], r["ldb"], -0.5, r["C"], r["ldc"])
        assert info == 0
        nviol, ratio = oracle.bound_violations(r["out_st"][:, :m], Cref, G, k, oracle.U64)
        assert nviol == 0, (m, n, k, ratio)
        assert np.array_equal(r["out_st"][:, m:], r["C"][:, m:], equal_nan=True)


def test_static_scratch_entry_refuses_what_the_array_cannot_hold():
    torch = torch_mod()
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)
    rng = si.rng_for(97, 1)
    m, n, k = 1280, 1280, 8192       # 100 tail tiles x 5 pieces x 128 KiB = 62.5 MiB
    plan = xg.xgemm_plan("d", 0, m, n, k, xg.xgemm_workspace_bytes())
    assert plan[1] > 1
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "N", m, n, k)
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    assert xg.xgemm_dgemm_static("N", "N", m, n, k, 1.0, dA, lda, dB, ldb, 0.0, dC, ldc) == xg.E_SCRATCH
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C, equal_nan=True)        # nothing was enqueued
    # argument errors come first, as in the other entry points
    assert xg.xgemm_dgemm_static("N", "N", m, n, k, 1.0, dA, m - 1, dB, ldb, 0.0, dC, ldc) == -8
    # and the next call that fits works
    m, n, k = 512, 512, 2048
    A, lda, B, ldb, C, ldc = make_operands(rng, "N", "N", m, n, k)
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    assert xg.xgemm_dgemm_static("N", "N", m, n, k, -1.0, dA, lda, dB, ldb, 1.0, dC, ldc) == 0
    torch.cuda.synchronize()
    info, Cref, G = oracle.gemm_ext("N", "N", m, n, k, -1.0, A, lda, B, ldb, 1.0, C, ldc)
    assert oracle.bound_violations(dC.cpu().numpy(), Cref, G, k, oracle.U64)[0] == 0
