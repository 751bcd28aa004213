"""The library's model functions (C ABI, host only) against the Python oracle
of the paper's formulas, on the paper's own tables and on random mixes; and
consistency of the CDNA4 instantiation with the tile geometry."""
import os
import random

import pytest

import paper_1611_08035_amd as xg
from oracle import queue_model as qm
from test_model_pins import rows


def test_outer_product_rate_matches_oracle_on_paper_tables():
    for perm, *_rest in rows("mic_prediction.txt"):
        mix = qm.xeon_phi_mix(int(perm))
        keys = sorted(mix)
        got = xg.xgemm_model_outer_product_rate([qm.XEON_PHI_RATES[k] for k in keys], [mix[k] for k in keys])
        assert got == qm.outer_product_rate(mix, qm.XEON_PHI_RATES)
    for _mr, _nr, _b, _s, l_mem, l_fma, l_shuf, _lam, _gf in rows("snb_prediction.txt"):
        mix = qm.sandy_bridge_mix(int(l_mem), int(l_fma), int(l_shuf))
        keys = sorted(mix)
        got = xg.xgemm_model_outer_product_rate([qm.SANDY_BRIDGE_RATES[k] for k in keys], [mix[k] for k in keys])
        assert got == qm.outer_product_rate(mix, qm.SANDY_BRIDGE_RATES)
    assert xg.xgemm_model_outer_product_rate([2, 1, 1, 1], [5, 4, 4, 4]) == 0.25   # Sec. 4.3 worked example


def test_random_mixes_and_stalls_match_oracle():
    rnd = random.Random(16110835)
    for _ in range(200):
        n = rnd.randint(1, 6)
        rate = [rnd.choice([0.5, 1.0, 2.0, 4.0]) for _ in range(n)]
        cnt = [rnd.choice([0, 1, 2, 3, 5, 8, 13, 30]) for _ in range(n)]
        want = qm.outer_product_rate({i: c for i, c in enumerate(cnt)}, {i: r for i, r in enumerate(rate)})
        assert xg.xgemm_model_outer_product_rate(rate, cnt) == want
        L, nd, k = rnd.randint(1, 40), rnd.randint(0, 5), rnd.randint(1, 9)
        assert xg.xgemm_model_stalled_rate(L, nd, k) == pytest.approx(qm.stalled_instruction_rate(L, nd, k), rel=1e-15)


def test_n_updates_matches_oracle_and_table():
    for name, r_total, v, m_r, n_r, r_r, want, *_ in rows("machine_table.txt"):
        args = (int(r_total), int(m_r), int(n_r), int(v))
        assert xg.xgemm_model_n_updates(*args, 0, int(r_r)) == qm.n_updates(*args, int(r_r)) == int(want), name
    assert xg.xgemm_model_n_updates(16, 4, 4, 0, 0, 1) == -1


@pytest.mark.parametrize("prec,es,mi,ki", [("d", 8, 16, 4), ("s", 4, 32, 2)])
def test_cdna4_instantiation_is_consistent_with_tile_geometry(prec, es, mi, ki):
    v = 0
    while xg.xgemm_variant_name(prec, v) is not None:
        name = xg.xgemm_variant_name(prec, v)
        mt_m, mt_n, kt = (int(x) for x in name.split("_")[1].split("x"))
        wgm, wgn = (int(x) for x in name.split("_")[2][1:].split("x"))
        for ta, tb in (("N", "N"), ("T", "N"), ("N", "T"), ("T", "T")):
            rc, o = xg.xgemm_model_predict(prec, v, ta, tb)
            assert rc == 0, name
            waves = wgm * wgn
            # MFMA flops of one slab of the macro-tile
            assert o[0] * waves * 2 * mi * mi * ki == 2 * mt_m * mt_n * kt
            # bytes staged per slab: global loads of 16 bytes per lane
            assert o[1] * waves * 64 * 16 == (mt_m + mt_n) * kt * es
            # LDS writes: 16 bytes per lane for an MN-contiguous operand, one element for a K-contiguous one
            assert o[3] >= o[1] and (o[3] == o[1]) == (ta == "N" and tb == "T")
            assert 0.5 < o[9] <= 1.0 and o[10] * o[11] <= 512
            assert o[4] >= o[5] and o[4] >= o[6]     # every variant is matrix-pipe bound
        v += 1
    assert v >= 5
    assert xg.xgemm_model_predict(prec, 99)[0] == -2 and xg.xgemm_model_predict("x", 0)[0] == -1


def _variants(prec):
    v = 0
    while xg.xgemm_variant_name(prec, v) is not None:
        yield v, xg.xgemm_variant_name(prec, v)
        v += 1


# Variants whose measured full-occupancy efficiency the model misses by more than the planner's tolerance;
# for these the planner keeps the measured figure.  s_128x128x32: the model sees a slab of twice the depth
# hide the barrier twice as well (0.97), the device runs it at 0.88.
MODEL_EXCEPTIONS = {"s_128x128x32_w2x2"}
MODEL_TOLERANCE = 0.025


@pytest.mark.parametrize("prec", ["d", "s"])
def test_model_efficiency_reproduces_the_measured_table(prec):
    table = {}
    for v, name in _variants(prec):
        rc, (measured, model, used) = xg.xgemm_model_efficiency(prec, v)
        assert rc == 0
        table[name] = (measured, model)
        if name in MODEL_EXCEPTIONS:
            assert abs(model - measured) > MODEL_TOLERANCE, name + " is no exception any more: take it off the list"
            assert used == pytest.approx(measured, abs=1e-7)
        else:
            assert abs(model - measured) <= MODEL_TOLERANCE, (name, measured, model)
            assert used == model
    # predicted order = measured order wherever the measurements tell two variants apart
    names = [n for n in table if n not in MODEL_EXCEPTIONS]
    told_apart = 0
    for a in names:
        for b in names:
            if table[a][0] - table[b][0] > MODEL_TOLERANCE:
                assert table[a][1] > table[b][1], (a, b, table[a], table[b])
                told_apart += 1
    assert told_apart >= 4
    assert MODEL_EXCEPTIONS & set(table) or prec == "d"


@pytest.mark.parametrize("prec", ["d", "s"])
def test_model_utilisation_is_the_papers_two_formulas(prec):
    """out[9] recomputed by the oracle from the counts the library reports: Sec. 4.3's stalled rate on the
    matrix pipe (one stall per workgroup on the CU), Sec. 4.2's minimum over the three pipelines."""
    for v, name in _variants(prec):
        wgm, wgn = (int(x) for x in name.split("_")[2][1:].split("x"))
        for ta, tb in (("N", "N"), ("T", "T")):
            rc, o = xg.xgemm_model_predict(prec, v, ta, tb)
            wgs = o[11] * 4 / (wgm * wgn)
            assert wgs == int(wgs) and wgs >= 1
            w_mfma = qm.stalled_wait(o[4], wgs, o[8] / wgs)
            assert w_mfma == pytest.approx(o[4] + o[8], rel=1e-15)
            want = o[4] * qm.outer_product_rate({"mfma": w_mfma, "lds": o[5], "vmem": o[6]},
                                                {"mfma": 1.0, "lds": 1.0, "vmem": 1.0})
            assert o[9] == pytest.approx(want, rel=1e-14), name
            assert o[9] == pytest.approx(qm.stalled_instruction_rate(o[4], wgs, o[8] / wgs), rel=1e-14)


@pytest.mark.parametrize("prec,es,tiles", [("d", 8, (16,)), ("s", 4, (32, 16))])
def test_design_space_enumeration(prec, es, tiles):
    cnt, rows = xg.xgemm_model_enumerate(prec, 4096)
    assert cnt == len(rows) and cnt > 100
    seen = set()
    for mi, wt_m, wt_n, wgm, wgn, kt, regs, lds, wgs, util, mt_m, mt_n in rows:
        assert mi in tiles and kt in (8, 16, 32) and wt_m % mi == 0 and wt_n % mi == 0
        assert (mt_m, mt_n) == (wt_m * wgm, wt_n * wgn)
        waves = wgm * wgn
        # Sec. 5.4: accumulators (wave tile / 64 lanes, in 32-bit registers) + something for the operands fit
        # the 512 registers a SIMD lane has, at the occupancy the row assumes
        acc = wt_m * wt_n * es // 4 // 64
        assert acc < regs <= 512
        assert 1 <= wgs <= 8 and regs * (wgs * waves / 4.0) <= 512 or waves < 4
        assert lds == 2 * kt * (mt_m + mt_n + 2 * (16 // es)) * es and lds * wgs <= 160 * 1024
        assert 0.0 < util < 1.0
        seen.add((int(mi), int(mt_m), int(mt_n), int(kt), int(wgm), int(wgn)))
    assert len(seen) == cnt
    assert [r[9] for r in rows] == sorted((r[9] for r in rows), reverse=True)
    # every built variant is a point of the space, and the enumeration gives it the utilisation predict() does
    by_key = {(int(r[0]), int(r[10]), int(r[11]), int(r[5]), int(r[3]), int(r[4])): r for r in rows}
    for v, name in _variants(prec):
        mt_m, mt_n, kt = (int(x) for x in name.split("_")[1].split("x"))
        wgm, wgn = (int(x) for x in name.split("_")[2][1:].split("x"))
        row = by_key[(tiles[0], mt_m, mt_n, kt, wgm, wgn)]
        rc, o = xg.xgemm_model_predict(prec, v)
        assert row[6] == o[10]
        if row[8] * wgm * wgn / 4 == o[11]:
            assert row[9] == pytest.approx(o[9], rel=1e-14)
    # the head of the list: a tile no smaller than the largest that is built, and the truncated call agrees
    cnt2, head = xg.xgemm_model_enumerate(prec, 5)
    assert cnt2 == cnt and head == rows[:5]
    assert xg.xgemm_model_enumerate(prec, 0)[0] == cnt
    assert xg.xgemm_model_enumerate("x", 4)[0] == -1
