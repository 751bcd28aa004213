"""Oracle for the paper's analytical kernel-selection model (Sec. 4 and 5.4).

TEST INFRASTRUCTURE ONLY, like the rest of ``oracle/``: plain Python written
from the paper's formulas, pinned by the tables the paper prints
(``tests/golden/*.txt``).  The library's own model (``xgemm_model_*`` in the C
ABI) is compared against it; the two share no code.

Formulas (own words):
  * Sec. 4.1-4.2: pipelines are queues, functional units are servers.  If an
    outer product puts L_i instructions into pipeline i and that pipeline
    retires lambda_i instructions per cycle, the outer-product rate is
    min_i lambda_i / L_i  (the slowest pipeline clears last).
  * Sec. 4.3: a pipeline holding n dependent instructions of latency k cannot
    hide that latency; its time per outer product grows from L to W = L + n k
    and, by Little's law, it sustains lambda = L / W instructions per cycle.
  * Sec. 6.1: flop/cycle = rate * m_r * n_r * 2;  GFLOP/s = f[GHz] * flop/cycle.
  * Sec. 5.4: N_updates = floor((R_total - m_r n_r / v - R_A) / R_R) and the
    sub-block must satisfy m_s n_s <= N_updates v.
"""
from __future__ import annotations

import math


def outer_product_rate(counts, rates):
    """min over pipelines of rates[p] / counts[p]; pipelines with no work are skipped."""
    best = math.inf
    for p, L in counts.items():
        if L > 0:
            best = min(best, rates[p] / L)
    return best


def stalled_wait(L, n_dependent, latency):
    """Time a pipeline needs for its L instructions when n of them expose their latency."""
    return L + n_dependent * latency


def stalled_instruction_rate(L, n_dependent, latency):
    """Little's law on the stalled pipeline: instructions per cycle."""
    return L / stalled_wait(L, n_dependent, latency)


def flop_per_cycle(rate, m_r, n_r):
    return rate * m_r * n_r * 2


def gflops(freq_ghz, fpc):
    return freq_ghz * fpc


def n_updates(r_total, m_r, n_r, v, r_r, r_a=None):
    if r_a is None:
        r_a = math.ceil(m_r / v)
    return math.floor((r_total - m_r * n_r / v - r_a) / r_r)


def subblock_fits(m_s, n_s, n_upd, v):
    return m_s * n_s <= n_upd * v


# ---- the paper's two validation families -------------------------------------------------
def xeon_phi_mix(permute_updates):
    """8 x 30 outer product from p permute unit updates (8 x 4: one load, one
    permute, four FMAs) and 30 - 4p broadcast unit updates (8 x 1: one load,
    one FMA), plus one load of a and four prefetches on the memory port.
    The table's vector-port column is one higher than that recipe gives
    (31 + p, not 30 + p); the extra instruction is taken to be the vector load
    of the column of a, which the text does not assign to a port."""
    bcast = 30 - 4 * permute_updates
    return {"mem": 1 + permute_updates + bcast + 4, "p0": 1 + permute_updates + 4 * permute_updates + bcast}


XEON_PHI_RATES = {"mem": 1.0, "p0": 1.0}
SANDY_BRIDGE_RATES = {"mem": 2.0, "mul": 1.0, "add": 1.0, "shuf": 1.0}


def sandy_bridge_mix(l_mem, l_fma, l_shuf):
    """Multiply and add are separate instructions on separate ports, L_fma of each."""
    return {"mem": l_mem, "mul": l_fma, "add": l_fma, "shuf": l_shuf}
