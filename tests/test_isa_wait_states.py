"""Regression guard for a wrong result that an earlier form of the order-256 product kernel gave for a few
orders, in some waves of some runs only: runtime jumps around whole accumulator tiles, each placed straight
after a tile's matrix instruction and all landing on one block that copies accumulator registers.  On the path
that jumps, the compiler had put fewer wait states between the matrix instruction and the copy of the register
pair it writes last than it puts everywhere else (14 against 19 in a rebuilt copy of that form), because its
search for the nearest matrix instruction visits each block once and reached those blocks first along the long
way round.  The fix was straight-line tile code.  This test compiles the level-3 kernels as the library build does
and checks on EVERY path that no reader of a double-precision matrix result comes sooner than the distance the
toolchain itself uses on the straight path."""
import os
import shutil
import subprocess
import tempfile

import pytest

from isa_walk import kernels, shortest_reads
from paper_1611_08035_amd import build as hip_build

# 16 passes of the 16x16x4 double-precision matrix instruction on this target plus 3: what the toolchain keeps
# between such an instruction and a vector instruction that reads its result wherever it sees the pair
DGEMM_RESULT_WAIT_STATES = 19


def test_no_path_reads_a_matrix_result_too_early():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    src = os.path.join(hip_build.CSRC, "xgemm_l3.hip")
    with tempfile.TemporaryDirectory() as td:
        out = os.path.join(td, "l3.s")
        cmd = [hipcc] + hip_build.HIPCC_FLAGS + hip_build.EXTRA_FLAGS.get("xgemm_l3.hip", []) + \
              ["--cuda-device-only", "-S", src, "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(out).read()
    ks = kernels(text)
    checked = 0
    for name, (ins, labels) in ks.items():
        hits = shortest_reads(ins, labels, "v_mfma_f64_16x16x4", limit=DGEMM_RESULT_WAIT_STATES + 1)
        checked += sum(1 for t in ins if t.startswith("v_mfma_f64_16x16x4"))
        for w, mma, reader in hits:
            assert w >= DGEMM_RESULT_WAIT_STATES, f"{name}: `{reader}` reads the result of `{mma}` after {w} wait states"
    assert checked > 500, "the level-3 kernels hold hundreds of double-precision matrix instructions"
