"""Pins for the queueing-model oracle: the numbers the paper prints
(tests/golden/*.txt, each with its citation) and the worked example of Sec. 4.3."""
import os

import pytest

from oracle import queue_model as qm

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def rows(name):
    out = []
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            out.append(line.split())
    return out


def test_worked_example_sandy_bridge_4x4():
    # Sec. 4.3: one load of a + four loads of b, four multiplies, four adds, four shuffles
    rate = qm.outer_product_rate({"mem": 5, "mul": 4, "add": 4, "shuf": 4}, qm.SANDY_BRIDGE_RATES)
    assert rate == 0.25
    # the memory pipeline alone would allow 2/5
    assert qm.outer_product_rate({"mem": 5}, qm.SANDY_BRIDGE_RATES) == pytest.approx(0.4)


def test_xeon_phi_table():
    for perm, bcast, l_mem, l_p0, lam, fpc, gf in rows("mic_prediction.txt"):
        mix = qm.xeon_phi_mix(int(perm))
        assert 30 - 4 * int(perm) == int(bcast)
        assert mix == {"mem": int(l_mem), "p0": int(l_p0)}
        rate = qm.outer_product_rate(mix, qm.XEON_PHI_RATES)
        assert rate == pytest.approx(float(lam), abs=6e-6)
        assert qm.flop_per_cycle(rate, 8, 30) == pytest.approx(float(fpc), abs=6e-3)
        assert qm.gflops(1.053, qm.flop_per_cycle(rate, 8, 30)) == pytest.approx(float(gf), abs=0.05)


def test_xeon_phi_best_mix_is_one_permute():
    rates = [qm.outer_product_rate(qm.xeon_phi_mix(p), qm.XEON_PHI_RATES) for p in range(8)]
    assert max(range(8), key=lambda p: rates[p]) == 1


def test_sandy_bridge_table():
    for m_r, n_r, _b, _s, l_mem, l_fma, l_shuf, lam, gf in rows("snb_prediction.txt"):
        rate = qm.outer_product_rate(qm.sandy_bridge_mix(int(l_mem), int(l_fma), int(l_shuf)),
                                     qm.SANDY_BRIDGE_RATES)
        assert rate == pytest.approx(float(lam), abs=6e-4)
        assert qm.gflops(3.3, qm.flop_per_cycle(rate, int(m_r), int(n_r))) == pytest.approx(float(gf), abs=0.05)


def test_n_updates_table():
    for name, r_total, v, m_r, n_r, r_r, want, m_s, n_s, flag in rows("machine_table.txt"):
        got = qm.n_updates(int(r_total), int(m_r), int(n_r), int(v), int(r_r))
        assert got == int(want), name
        assert qm.subblock_fits(int(m_s), int(n_s), got, int(v)) == (flag == "ok"), name


def test_stall_correction():
    # no dependent instructions: the pipeline runs at one instruction per cycle
    assert qm.stalled_instruction_rate(8, 0, 5) == 1.0
    # 4 instructions, 2 of which expose a latency of 3: W = 4 + 6
    assert qm.stalled_wait(4, 2, 3) == 10 and qm.stalled_instruction_rate(4, 2, 3) == pytest.approx(0.4)
