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
