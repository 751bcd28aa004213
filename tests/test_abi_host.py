"""Host-side checks that need no GPU: the shared library loads, exports every
symbol the header declares, and rejects illegal arguments before touching a
device."""
import os
import re

import pytest

import paper_1611_08035_amd as xg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


HEADERS = ("xgemm.h", "xgemm_tuning.h", "xgemm_probe.h")


def declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(xgemm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = xg.lib()
    names = []
    for header in HEADERS:
        mine = declared_symbols(header)
        assert len(mine) >= 4, header
        for name in mine:
            assert hasattr(L, name), f"{name} declared in {header} but not exported"
            assert name not in names, f"{name} declared in two headers"
        names += mine
    assert sorted(xg.EXPORTS) == sorted(names)


def test_blas_header_leads_with_the_hot_path_and_holds_no_controls():
    """The six calls of the hot path come first in xgemm.h; benchmark controls, the planner, the model and
    the probes live in the two other headers."""
    blas = declared_symbols("xgemm.h")
    text = open(os.path.join(ROOT, "include", "xgemm.h")).read()
    order = [m.group(1) for m in re.finditer(r"^(?:int|size_t|const char \*)\s*\*?(xgemm_[a-z0-9_]+)\(", text, flags=re.M)]
    assert order[:6] == ["xgemm_dgemm", "xgemm_sgemm", "xgemm_zgemm_split", "xgemm_zgemm_worksize", "xgemm_version",
                         "xgemm_last_kernel_name"]
    for name in blas:
        assert not any(w in name for w in ("force", "probe", "model", "plan", "tile_map", "variant")), name
    assert "xgemm_tuning_reset" in declared_symbols("xgemm_tuning.h")


def test_tuning_controls_are_sticky_until_reset():
    """A forced variant or split stays in force on the calling thread until it is set back or everything is reset."""
    full = xg.xgemm_workspace_bytes()
    auto = xg.xgemm_plan("d", 0, 4096, 4096, 4096, full)
    assert xg.xgemm_force_variant(3) == 0 and xg.xgemm_force_split(0) == 0
    assert xg.xgemm_force_potrf_panel(512) == 0 and xg.xgemm_force_potrf_block(64) == 0
    assert xg.xgemm_plan("d", 0, 4096, 4096, 4096, full)[0] == 3
    assert xg.xgemm_plan("d", 0, 4096, 4096, 4096, full)[0] == 3          # still
    xg.xgemm_tuning_reset()
    assert xg.xgemm_plan("d", 0, 4096, 4096, 4096, full) == auto


def test_version_and_variant_names():
    assert "gfx950" in xg.xgemm_version()
    assert xg.xgemm_variant_name("d", 0).startswith("d_")
    assert xg.xgemm_variant_name("s", 0).startswith("s_")
    assert xg.xgemm_variant_name("d", 1000) is None
    assert xg.xgemm_force_variant(1000) == -1
    assert xg.xgemm_force_variant(-1) == 0


@pytest.mark.parametrize("fn", ["xgemm_dgemm", "xgemm_sgemm"])
def test_illegal_arguments_are_rejected_on_the_host(fn):
    f = getattr(xg, fn)
    P = 4096   # any non-null address: nothing is launched on an error path
    g = lambda *a: f(*a, stream=0)
    assert g("X", "N", 2, 2, 2, 1.0, P, 2, P, 2, 0.0, P, 2) == -1
    assert g("N", "Q", 2, 2, 2, 1.0, P, 2, P, 2, 0.0, P, 2) == -2
    assert g("N", "N", -1, 2, 2, 1.0, P, 2, P, 2, 0.0, P, 2) == -3
    assert g("N", "N", 2, -1, 2, 1.0, P, 2, P, 2, 0.0, P, 2) == -4
    assert g("N", "N", 2, 2, -1, 1.0, P, 2, P, 2, 0.0, P, 2) == -5
    assert g("N", "N", 2, 2, 2, 1.0, None, 2, P, 2, 0.0, P, 2) == -7
    assert g("N", "N", 3, 2, 2, 1.0, P, 2, P, 2, 0.0, P, 3) == -8
    assert g("T", "N", 3, 2, 4, 1.0, P, 3, P, 4, 0.0, P, 3) == -8
    assert g("N", "N", 2, 2, 2, 1.0, P, 2, None, 2, 0.0, P, 2) == -9
    assert g("N", "N", 2, 2, 3, 1.0, P, 2, P, 2, 0.0, P, 2) == -10
    assert g("N", "T", 2, 3, 2, 1.0, P, 2, P, 2, 0.0, P, 2) == -10
    assert g("N", "N", 2, 2, 2, 1.0, P, 2, P, 2, 0.0, None, 2) == -12
    assert g("N", "N", 3, 2, 2, 1.0, P, 3, P, 2, 0.0, P, 2) == -13
    assert g("N", "N", 0, 2, 2, 1.0, P, 0, P, 2, 0.0, P, 1) == -8
    assert g("N", "N", 2 ** 31, 2, 2, 1.0, P, 2 ** 31, P, 2, 0.0, P, 2 ** 31) == -3
    # quick returns launch nothing and succeed
    assert g("N", "N", 0, 2, 2, 1.0, None, 1, None, 2, 0.0, None, 1) == 0
    assert g("N", "N", 2, 0, 2, 1.0, None, 2, None, 2, 0.0, None, 2) == 0
    assert g("N", "N", 2, 2, 0, 1.0, None, 2, None, 1, 1.0, P, 2) == 0
    assert g("N", "N", 2, 2, 2, 0.0, None, 2, None, 2, 1.0, P, 2) == 0
    assert xg.xgemm_last_kernel_name() == "none"


@pytest.mark.parametrize("fn", ["xgemm_dsyrk", "xgemm_ssyrk"])
def test_syrk_illegal_arguments_and_quick_returns(fn):
    f = getattr(xg, fn)
    P = 4096
    g = lambda *a: f(*a, stream=0)
    assert g("X", "N", 2, 2, 1.0, P, 2, 0.0, P, 2) == -1
    assert g("L", "Q", 2, 2, 1.0, P, 2, 0.0, P, 2) == -2
    assert g("L", "N", -1, 2, 1.0, P, 2, 0.0, P, 2) == -3
    assert g("L", "N", 2 ** 31, 2, 1.0, P, 2 ** 31, 0.0, P, 2 ** 31) == -3
    assert g("U", "N", 2, -1, 1.0, P, 2, 0.0, P, 2) == -4
    assert g("U", "N", 2, 2, 1.0, None, 2, 0.0, P, 2) == -6
    assert g("L", "N", 3, 2, 1.0, P, 2, 0.0, P, 3) == -7
    assert g("L", "T", 2, 3, 1.0, P, 2, 0.0, P, 2) == -7
    assert g("L", "N", 2, 2, 1.0, P, 2, 0.0, None, 2) == -9
    assert g("L", "N", 3, 2, 1.0, P, 3, 0.0, P, 2) == -10
    assert g("L", "N", 0, 2, 1.0, None, 1, 0.0, None, 1) == 0
    assert g("U", "T", 2, 0, 1.0, None, 1, 1.0, P, 2) == 0
    assert g("U", "C", 2, 2, 0.0, None, 2, 1.0, P, 2) == 0
    assert xg.xgemm_last_kernel_name() == "none"


def test_zgemm_illegal_arguments_and_worksize():
    P = 4096
    z = lambda *a, **kw: xg.xgemm_zgemm_split(*a, stream=0, **kw)
    assert xg.xgemm_zgemm_worksize(5, 7, (1, 0), (0, 0)) == 0
    assert xg.xgemm_zgemm_worksize(5, 7, (1, 2), (0, 0)) == 70
    assert xg.xgemm_zgemm_worksize(5, 7, (1, 0), (0, 1)) == 70
    assert z("X", "N", 2, 2, 2, (1, 0), P, P, 2, P, P, 2, (0, 0), P, P, 2) == -1
    assert z("N", "N", 2, 2, 2, None, P, P, 2, P, P, 2, (0, 0), P, P, 2) == -6
    assert z("N", "N", 2, 2, 2, (1, 0), P, None, 2, P, P, 2, (0, 0), P, P, 2) == -8
    assert z("N", "N", 3, 2, 2, (1, 0), P, P, 2, P, P, 2, (0, 0), P, P, 3) == -9
    assert z("N", "N", 2, 2, 2, (1, 0), P, P, 2, None, P, 2, (0, 0), P, P, 2) == -10
    assert z("N", "N", 2, 2, 3, (1, 0), P, P, 2, P, P, 2, (0, 0), P, P, 2) == -12
    assert z("N", "N", 2, 2, 2, (1, 0), P, P, 2, P, P, 2, None, P, P, 2) == -13
    assert z("N", "N", 2, 2, 2, (1, 0), P, P, 2, P, P, 2, (0, 0), P, None, 2) == -15
    assert z("N", "N", 3, 2, 2, (1, 0), P, P, 3, P, P, 2, (0, 0), P, P, 2) == -16
    assert z("N", "N", 2, 2, 2, (1, 1), P, P, 2, P, P, 2, (0, 0), P, P, 2, work=None, lwork=8) == -17
    assert z("N", "N", 2, 2, 2, (1, 1), P, P, 2, P, P, 2, (0, 0), P, P, 2, work=P, lwork=7) == -18
    assert z("N", "N", 0, 2, 2, (1, 1), None, None, 1, None, None, 2, (0, 0), None, None, 1) == 0


@pytest.mark.parametrize("fn", ["xgemm_dtrsm", "xgemm_strsm", "xgemm_dtrmm", "xgemm_strmm"])
def test_trsm_illegal_arguments_and_quick_returns(fn):
    f = getattr(xg, fn)
    P = 4096
    g = lambda *a: f(*a, stream=0)
    assert g("X", "L", "N", "N", 4, 3, 1.0, P, 4, P, 4) == -1
    assert g("L", "X", "N", "N", 4, 3, 1.0, P, 4, P, 4) == -2
    assert g("L", "L", "X", "N", 4, 3, 1.0, P, 4, P, 4) == -3
    assert g("L", "L", "N", "X", 4, 3, 1.0, P, 4, P, 4) == -4
    assert g("L", "L", "N", "N", -1, 3, 1.0, P, 4, P, 4) == -5
    assert g("L", "L", "N", "N", 4, 2 ** 31, 1.0, P, 4, P, 4) == -6
    assert g("L", "L", "N", "N", 4, 3, 1.0, None, 4, P, 4) == -8
    assert g("L", "L", "N", "N", 4, 3, 1.0, P, 3, P, 4) == -9
    assert g("R", "L", "N", "N", 4, 3, 1.0, P, 2, P, 4) == -9
    assert g("L", "L", "N", "N", 4, 3, 1.0, P, 4, None, 4) == -10
    assert g("L", "L", "N", "N", 4, 3, 1.0, P, 4, P, 3) == -11
    assert g("L", "L", "N", "N", 0, 3, 1.0, None, 1, None, 1) == 0
    assert g("R", "U", "T", "U", 4, 0, 1.0, None, 1, None, 4) == 0


@pytest.mark.parametrize("fn", ["xgemm_dpotrf", "xgemm_spotrf"])
def test_potrf_illegal_arguments(fn):
    f = getattr(xg, fn)
    P = 4096
    assert f("X", 4, P, 4, P, stream=0) == -1
    assert f("L", -1, P, 4, P, stream=0) == -2
    assert f("L", 2 ** 31, P, 2 ** 31, P, stream=0) == -2
    assert f("U", 4, None, 4, P, stream=0) == -3
    assert f("U", 4, P, 3, P, stream=0) == -4
    assert f("L", 4, P, 4, None, stream=0) == -5


@pytest.mark.parametrize("fn", ["xgemm_dgetrf", "xgemm_sgetrf"])
def test_getrf_illegal_arguments(fn):
    f = getattr(xg, fn)
    P = 4096                                       # never dereferenced: every call below is refused on the host
    assert f(-1, 4, P, 4, P, P, stream=0) == -1
    assert f(4, -1, P, 4, P, P, stream=0) == -2
    assert f(4, 4, None, 4, P, P, stream=0) == -3
    assert f(5, 4, P, 4, P, P, stream=0) == -4
    assert f(4, 4, P, 4, None, P, stream=0) == -5
    assert f(4, 4, P, 4, P, None, stream=0) == -6
    assert xg.xgemm_force_getrf_panel(0) == -1 and xg.xgemm_force_getrf_panel(-2) == -1
    assert xg.xgemm_force_getrf_panel(64) == 0 and xg.xgemm_force_getrf_panel(-1) == 0
    # the routine with an exchange buffer: the same numbering, then the buffer's alignment
    w = getattr(xg, fn + "_ws")
    lw = xg.xgemm_getrf_workspace_bytes()
    assert 0 < lw <= 2 << 20
    assert w(-1, 4, P, 4, P, P, P, lw, stream=0) == -1
    assert w(5, 4, P, 4, P, P, P, lw, stream=0) == -4
    assert w(4, 4, P, 4, P, None, P, lw, stream=0) == -6
    assert w(4, 4, P, 4, P, P, P + 8, lw, stream=0) == -7
    assert xg.xgemm_force_getrf_spin_limit(-1) == -1 and xg.xgemm_force_getrf_spin_limit(5) == 0
    assert xg.xgemm_force_getrf_poll_delay(-1, 0) == -1 and xg.xgemm_force_getrf_poll_delay(0, 2000) == -1
    assert xg.xgemm_force_getrf_poll_delay(4, 4) == 0
    assert xg.xgemm_force_getrf_shared(1) == -1 and xg.xgemm_force_getrf_shared(0) == 0 and xg.xgemm_force_getrf_shared(-1) == 0
    xg.xgemm_tuning_reset()


@pytest.mark.parametrize("pre", "ds")
def test_syr2k_and_symm_illegal_arguments(pre):
    P = 4096
    f = getattr(xg, f"xgemm_{pre}syr2k")
    g = lambda *a: f(*a, stream=0)
    assert g("X", "N", 4, 3, 1.0, P, 4, P, 4, 0.0, P, 4) == -1
    assert g("L", "X", 4, 3, 1.0, P, 4, P, 4, 0.0, P, 4) == -2
    assert g("L", "N", -1, 3, 1.0, P, 4, P, 4, 0.0, P, 4) == -3
    assert g("L", "N", 4, -1, 1.0, P, 4, P, 4, 0.0, P, 4) == -4
    assert g("L", "N", 4, 3, 1.0, None, 4, P, 4, 0.0, P, 4) == -6
    assert g("L", "N", 4, 3, 1.0, P, 3, P, 4, 0.0, P, 4) == -7
    assert g("L", "N", 4, 3, 1.0, P, 4, None, 4, 0.0, P, 4) == -8
    assert g("L", "T", 4, 3, 1.0, P, 3, P, 2, 0.0, P, 4) == -9
    assert g("L", "N", 4, 3, 1.0, P, 4, P, 4, 0.0, None, 4) == -11
    assert g("L", "N", 4, 3, 1.0, P, 4, P, 4, 0.0, P, 3) == -12
    assert g("U", "T", 0, 3, 1.0, None, 3, None, 3, 0.0, None, 1) == 0
    assert g("U", "N", 4, 0, 1.0, None, 4, None, 4, 1.0, P, 4) == 0
    f = getattr(xg, f"xgemm_{pre}symm")
    g = lambda *a: f(*a, stream=0)
    assert g("X", "L", 4, 3, 1.0, P, 4, P, 4, 0.0, P, 4) == -1
    assert g("L", "X", 4, 3, 1.0, P, 4, P, 4, 0.0, P, 4) == -2
    assert g("L", "L", -1, 3, 1.0, P, 4, P, 4, 0.0, P, 4) == -3
    assert g("L", "L", 4, -1, 1.0, P, 4, P, 4, 0.0, P, 4) == -4
    assert g("L", "L", 4, 3, 1.0, None, 4, P, 4, 0.0, P, 4) == -6
    assert g("L", "L", 4, 3, 1.0, P, 3, P, 4, 0.0, P, 4) == -7
    assert g("R", "L", 4, 3, 1.0, P, 2, P, 4, 0.0, P, 4) == -7
    assert g("L", "L", 4, 3, 1.0, P, 4, None, 4, 0.0, P, 4) == -8
    assert g("L", "L", 4, 3, 1.0, P, 4, P, 3, 0.0, P, 4) == -9
    assert g("L", "L", 4, 3, 1.0, P, 4, P, 4, 0.0, None, 4) == -11
    assert g("L", "L", 4, 3, 1.0, P, 4, P, 4, 0.0, P, 3) == -12
    assert g("L", "L", 0, 3, 1.0, None, 1, None, 1, 0.0, None, 1) == 0
    assert g("R", "U", 4, 3, 0.0, None, 3, None, 4, 1.0, P, 4) == 0


def test_workspace_routines_host_side():
    P = 4096
    assert xg.xgemm_workspace_bytes() == 8192 + (64 << 20)
    assert xg.xgemm_workspace_init(None, 1 << 20, stream=0) == -1
    assert xg.xgemm_workspace_init(P + 4, 1 << 20, stream=0) == -1
    assert xg.xgemm_workspace_init(P, 100, stream=0) == -2
    for f in (xg.xgemm_dgemm_ws, xg.xgemm_sgemm_ws):
        assert f("X", "N", 2, 2, 2, 1.0, P, 2, P, 2, 0.0, P, 2, P, 1 << 20, stream=0) == -1
        assert f("N", "N", 3, 2, 2, 1.0, P, 3, P, 2, 0.0, P, 2, P, 1 << 20, stream=0) == -13
        assert f("N", "N", 2, 2, 2, 1.0, P, 2, P, 2, 0.0, P, 2, P + 8, 1 << 20, stream=0) == -14
        assert f("N", "N", 0, 2, 2, 1.0, None, 1, None, 2, 0.0, None, 1, None, 0, stream=0) == 0
    for f in (xg.xgemm_dsyrk_ws, xg.xgemm_ssyrk_ws):
        assert f("X", "N", 2, 2, 1.0, P, 2, 0.0, P, 2, P, 1 << 20, stream=0) == -1
        assert f("L", "N", 3, 2, 1.0, P, 3, 0.0, P, 2, P, 1 << 20, stream=0) == -10
        assert f("L", "N", 2, 2, 1.0, P, 2, 0.0, P, 2, P + 4, 1 << 20, stream=0) == -11
        assert f("L", "N", 0, 2, 1.0, None, 1, 0.0, None, 1, None, 0, stream=0) == 0
    assert xg.xgemm_force_split(33) == -1 and xg.xgemm_force_split(-2) == -1 and xg.xgemm_force_split(1) == 0
    assert xg.xgemm_force_split(4) == 0 and xg.xgemm_force_split(0) == 0 and xg.xgemm_force_split(-1) == 0
    assert xg.xgemm_last_split() == 1
    assert xg.xgemm_force_potrf_panel(-2) == -1 and xg.xgemm_force_potrf_panel(512) == 0 and xg.xgemm_force_potrf_panel(0) == 0
    assert xg.xgemm_force_potrf_panel(-1) == 0
    assert xg.xgemm_force_potrf_block(100) == -1 and xg.xgemm_force_potrf_block(128) == 0 and xg.xgemm_force_potrf_block(-1) == 0


@pytest.mark.parametrize("mt_m,mt_n", [(128, 128), (256, 128), (64, 64), (128, 64), (64, 128)])
@pytest.mark.parametrize("uplo", [0, 1, 2])
def test_tile_order_covers_every_needed_tile_exactly_once(uplo, mt_m, mt_n):
    for m, n in [(1, 1), (100, 100), (1000, 1000), (8192, 8192), (4097, 4097), (3001, 3001)] + \
            ([(4097, 3001), (130, 9000), (9000, 130)] if uplo == 0 else []):
        cnt, tiles = xg.xgemm_tile_map(uplo, m, n, mt_m, mt_n)
        ntm, ntn = -(-m // mt_m), -(-n // mt_n)
        assert cnt == len(tiles) and len(set(tiles)) == cnt, "a tile is visited twice"
        assert all(0 <= tm < ntm and 0 <= tn < ntn for tm, tn in tiles)
        def needed(tm, tn):
            r0, r1 = tm * mt_m, min(m, (tm + 1) * mt_m) - 1
            c0, c1 = tn * mt_n, min(n, (tn + 1) * mt_n) - 1
            return True if uplo == 0 else (r1 >= c0 if uplo == 1 else c1 >= r0)
        need = {(tm, tn) for tm in range(ntm) for tn in range(ntn) if needed(tm, tn)}
        assert need == set(tiles), "the order must hold exactly the tiles of the requested part of C"


def test_tile_order_xcd_runs_are_contiguous():
    # workgroups b = x (mod 8) share an XCD; each XCD must own one contiguous run of the band order
    cnt, tiles = xg.xgemm_tile_map(0, 8192, 8192, 128, 128)
    order = {t: i for i, t in enumerate(
        (first + r, c) for first in range(0, 64, 8) for c in range(64) for r in range(8))}
    for x in range(8):
        pos = [order[tiles[b]] for b in range(x, cnt, 8)]
        assert pos == list(range(pos[0], pos[0] + len(pos)))
    assert xg.xgemm_tile_map(3, 8, 8, 8, 8)[0] == -1 and xg.xgemm_tile_map(0, 0, 8, 8, 8)[0] == -2
    assert xg.xgemm_tile_map(0, 8, 8, 0, 8)[0] == -4


def test_interleaved_zgemm_illegal_arguments_and_work_size():
    P = 4096
    z = lambda *a, **kw: xg.xgemm_zgemm(*a, stream=0, **kw)
    assert xg.xgemm_zgemm_workbytes(5, 7, 3, 0) == 8 * 2 * (15 + 21 + 35)
    assert xg.xgemm_zgemm_workbytes(5, 7, 3, 1) == 8 * 3 * (15 + 21 + 35)
    assert xg.xgemm_zgemm_workbytes(0, 7, 3, 0) == 0
    big = 1 << 20
    ok = dict(work=P, lwork=big)
    assert z("X", "N", 2, 2, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, **ok) == -1
    assert z("N", "X", 2, 2, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, **ok) == -2
    assert z("N", "N", -1, 2, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, **ok) == -3
    assert z("N", "N", 2, -1, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, **ok) == -4
    assert z("N", "N", 2, 2, -1, (1, 0), P, 2, P, 2, (0, 0), P, 2, **ok) == -5
    assert z("N", "N", 2, 2, 2, None, P, 2, P, 2, (0, 0), P, 2, **ok) == -6
    assert z("N", "N", 2, 2, 2, (1, 0), None, 2, P, 2, (0, 0), P, 2, **ok) == -7
    assert z("N", "N", 2, 2, 2, (1, 0), P + 8, 2, P, 2, (0, 0), P, 2, **ok) == -7
    assert z("C", "N", 2, 2, 3, (1, 0), P, 2, P, 3, (0, 0), P, 2, **ok) == -8
    assert z("N", "N", 2, 2, 2, (1, 0), P, 2, None, 2, (0, 0), P, 2, **ok) == -9
    assert z("N", "T", 2, 3, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, **ok) == -10
    assert z("N", "N", 2, 2, 2, (1, 0), P, 2, P, 2, None, P, 2, **ok) == -11
    assert z("N", "N", 2, 2, 2, (1, 0), P, 2, P, 2, (0, 0), None, 2, **ok) == -12
    assert z("N", "N", 3, 2, 2, (1, 0), P, 3, P, 2, (0, 0), P, 2, **ok) == -13
    assert z("N", "N", 2, 2, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, method=3, **ok) == -14
    assert z("N", "N", 2, 2, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, method=-1, **ok) == -14
    # the fused form packs a 2m x 2k and an n x 2k operand
    assert xg.xgemm_zgemm_workbytes(5, 7, 3, 2) == 8 * (xg.xgemm_pack_elems(10, 6) + xg.xgemm_pack_elems(7, 6)) == 8 * 2 * 256 * 32
    assert xg.xgemm_zgemm_workbytes(5, 7, 0, 2) == 0
    assert z("N", "N", 2, 2, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, method=2, work=P, lwork=8 * 2 * 256 * 32 - 1) == -16
    assert z("N", "N", 2, 2, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, work=None, lwork=big) == -15
    assert z("N", "N", 2, 2, 2, (1, 0), P, 2, P, 2, (0, 0), P, 2, work=P, lwork=8 * 2 * 12 - 1) == -16
    assert z("N", "N", 0, 2, 2, (1, 0), None, 1, None, 2, (0, 0), None, 1) == 0
    assert z("N", "N", 2, 2, 0, (1, 0), None, 2, None, 1, (1, 0), P, 2) == 0


def test_missing_library_raises(monkeypatch):
    import paper_1611_08035_amd.xgemm as mod
    monkeypatch.setattr(mod, "_lib", None)
    monkeypatch.setattr(mod, "_LIBPATH", "/nonexistent/libxgemm.so")
    with pytest.raises(mod.XgemmError):
        mod.lib()


def test_pack_argument_checks_and_sizes():
    """Host side of the packed-operand calls: sizes and the illegal-argument numbers of include/xgemm.h."""
    assert xg.xgemm_pack_elems(1, 1) == 256 * 32 and xg.xgemm_pack_elems(257, 33) == 512 * 64
    assert xg.xgemm_pack_elems(0, 5) == 0 and xg.xgemm_pack_elems(-1, 5) == 0
    one = 16      # a non-null address that is never dereferenced: every call below fails its checks first
    for f in (xg.xgemm_dpack_a, xg.xgemm_spack_a):
        assert f("X", 4, 4, one, 4, one, stream=0) == -1
        assert f("N", -1, 4, one, 4, one, stream=0) == -2
        assert f("N", 4, -1, one, 4, one, stream=0) == -3
        assert f("N", 4, 4, None, 4, one, stream=0) == -4
        assert f("N", 4, 6, one, 3, one, stream=0) == -5      # stored 4 x 6: lda >= 4
        assert f("T", 4, 6, one, 5, one, stream=0) == -5      # stored 6 x 4: lda >= 6
        assert f("N", 4, 4, one, 4, None, stream=0) == -6
    for f in (xg.xgemm_dpack_b, xg.xgemm_spack_b):
        assert f("N", 6, 4, one, 5, one, stream=0) == -5      # stored 6 x 4 (k x n): ldb >= 6
        assert f("T", 6, 4, one, 3, one, stream=0) == -5      # stored 4 x 6 (n x k): ldb >= 4
        assert f("N", 6, 4, one, 6, None, stream=0) == -6
    for f in (xg.xgemm_dgemm_packed, xg.xgemm_sgemm_packed):
        assert f(-1, 2, 2, 1.0, one, one, 0.0, one, 2, stream=0) == -1
        assert f(2, -1, 2, 1.0, one, one, 0.0, one, 2, stream=0) == -2
        assert f(2, 2, -1, 1.0, one, one, 0.0, one, 2, stream=0) == -3
        assert f(2, 2, 2, 1.0, None, one, 0.0, one, 2, stream=0) == -5
        assert f(2, 2, 2, 1.0, one, None, 0.0, one, 2, stream=0) == -6
        assert f(2, 2, 2, 1.0, one, one, 0.0, None, 2, stream=0) == -8
        assert f(2, 2, 2, 1.0, one, one, 0.0, one, 1, stream=0) == -9
        assert f(0, 2, 2, 1.0, None, None, 0.0, None, 1, stream=0) == 0
