"""The entry points only enqueue kernels on the caller's stream (no allocation,
no memset, no synchronisation), so a chain of them can be captured in a HIP
graph.  (The factorisation of large orders also uses a stream of the library's
that forks from and joins the caller's; tests/test_gpu_potrf.py captures that.)  A captured chain -- product, triangular update with workspace, solve,
factorisation -- is replayed several times with eager work in between; every
replay must reproduce the eager result bit for bit."""
import numpy as np
import pytest

import paper_1611_08035_amd as xg
import synth_inputs as si
from gpu_util import to_dev, torch_mod

pytestmark = pytest.mark.gpu


def test_captured_chain_replays_bit_identically():
    torch = torch_mod()
    xg.xgemm_force_variant(-1)
    xg.xgemm_force_split(-1)
    rng = si.rng_for(190, 0)
    n, k = 1100, 300
    A = to_dev(si.uniform(rng, n, k))
    T = to_dev(si.triangular(rng, n, n, np.float64, "L", False, sentinel=0.0))
    S0 = to_dev(si.spd(rng, n, n, np.float64, "L", sentinel=0.0))
    C0 = to_dev(si.uniform(rng, n, n))
    C, S = C0.clone(), S0.clone()
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    lw = xg.xgemm_workspace_bytes()
    work = torch.zeros(lw, dtype=torch.uint8, device="cuda")

    def chain():
        # C := -A A^T + C (general product), lower triangle again with the workspace routine,
        # C := T^-1 C, then the Cholesky factor of S and S := S L^-T ... all in place
        assert xg.xgemm_dgemm("N", "T", n, n, k, -1.0, A, n, A, n, 1.0, C, n) == 0
        assert xg.xgemm_dsyrk_ws("L", "N", n, k, 0.5, A, n, 1.0, C, n, work, lw) == 0
        assert xg.xgemm_dtrsm("L", "L", "N", "N", n, n, 1.0, T, n, C, n) == 0
        assert xg.xgemm_dpotrf("L", n, S, n, info) == 0
        assert xg.xgemm_dtrmm("R", "L", "T", "N", n, n, 2.0, S, n, C, n) == 0

    # eager reference (also warms every kernel up outside the capture)
    chain()
    torch.cuda.synchronize()
    want_C, want_S = C.clone(), S.clone()
    assert int(info.item()) == 0

    graph = torch.cuda.CUDAGraph()
    C.copy_(C0)
    S.copy_(S0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        chain()
    for rep in range(3):
        C.copy_(C0)
        S.copy_(S0)
        info.fill_(7)
        scratch = torch.rand(512, 512, device="cuda") @ torch.rand(512, 512, device="cuda")   # unrelated eager work
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, want_C) and torch.equal(S, want_S), f"replay {rep} differs from the eager run"
        assert int(info.item()) == 0
        del scratch


def test_captured_lu_with_shared_panels_replays_bit_identically():
    """xgemm_dgetrf_ws enqueues kernels only (the exchange buffer is cleared by a kernel, the workgroups of a
    panel wait for each other inside one kernel), so it can be captured too; every replay gives the eager bits."""
    torch = torch_mod()
    xg.xgemm_tuning_reset()
    rng = si.rng_for(191, 0)
    n = 1100
    A0 = to_dev(si.uniform(rng, n, n))
    A = A0.clone()
    piv = torch.zeros(n, dtype=torch.int32, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    lw = xg.xgemm_getrf_workspace_bytes()
    work = torch.empty(lw, dtype=torch.uint8, device="cuda")

    def step():
        assert xg.xgemm_dgetrf_ws(n, n, A, n, piv, info, work, lw) == 0

    step()
    torch.cuda.synchronize()
    want_A, want_piv = A.clone(), piv.clone()
    assert int(info.item()) == 0
    graph = torch.cuda.CUDAGraph()
    A.copy_(A0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        A.copy_(A0)
        piv.fill_(-3)
        info.fill_(7)
        work.fill_(rep)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(A, want_A) and torch.equal(piv, want_piv), f"replay {rep} differs from the eager run"
        assert int(info.item()) == 0


def test_captured_plain_lu_allocates_nothing_and_replays_bit_identically():
    """Under capture xgemm_dgetrf may neither allocate its exchange buffer nor wait for the library's event:
    panels of more than 128 rows go to the leaves of one workgroup each, the others stay in LDS.  The capture
    succeeds, every replay gives the same bits, and they are a valid factorisation."""
    import oracle
    from lu_util import check_valid
    torch = torch_mod()
    xg.xgemm_tuning_reset()
    rng = si.rng_for(192, 0)
    n = 700
    A_host = si.uniform(rng, n, n)
    A0 = to_dev(A_host)
    A = A0.clone()
    piv = torch.zeros(n, dtype=torch.int32, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        assert xg.xgemm_dgetrf(n, n, A, n, piv, info) == 0
    first = None
    for rep in range(3):
        A.copy_(A0)
        piv.fill_(-3)
        info.fill_(7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(info.item()) == 0
        got = (A.clone(), piv.clone())
        if first is None:
            first = got
        assert torch.equal(got[0], first[0]) and torch.equal(got[1], first[1]), f"replay {rep} differs from the first"
    check_valid(n, n, A_host, n, first[0].cpu().numpy(), n, first[1].cpu().numpy(), oracle.U64)
