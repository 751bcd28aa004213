"""Run as a script with XGEMM_REQUIRE_ALIGNED=1 in the environment (the library
reads it when it is loaded): operands with odd leading dimensions then take the
element-wise fallback kernels, which are checked here like any other variant."""
import itertools
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import oracle  # noqa: E402
import paper_1611_08035_amd as xg  # noqa: E402
import synth_inputs as si  # noqa: E402
from gpu_util import check_full, check_syrk_full, make_operands, make_syrk_operands, run_real  # noqa: E402


def main():
    assert os.environ.get("XGEMM_REQUIRE_ALIGNED"), "set XGEMM_REQUIRE_ALIGNED=1"
    for dtype, prec in ((np.float64, "d"), (np.float32, "s")):
        rng = si.rng_for(94, 0 if prec == "d" else 1)
        for (m, n, k), ta, tb in itertools.product([(300, 275, 83), (64, 64, 16), (1, 1, 1), (17, 130, 5)], "NT", "NT"):
            A, lda, B, ldb, C, ldc = make_operands(rng, ta, tb, m, n, k, (1, 3, 5), dtype)
            ratio = check_full(xg, ta, tb, m, n, k, 1.5, A, lda, B, ldb, -0.5, C, ldc)
            name = xg.xgemm_last_kernel_name()
            # 64x64: the fallback's tile; a case whose leading dimensions happen to be aligned takes the ordinary
            # path, where so small a product may get the 32x32 tile
            assert ("64x64" in name or "32x32" in name) and ratio < 1.0, (name, ratio)
            print(f"fallback {prec} {ta}{tb} {m}x{n}x{k} {name} ratio {ratio:.3f}", flush=True)
        R = 1000 if prec == "d" else 8
        A, lda, B, ldb, C, ldc = make_operands(rng, "T", "N", 200, 131, 300, (1, 1, 1), dtype, "int", R)
        out = run_real(xg, "T", "N", 200, 131, 300, 2.0, A, lda, B, ldb, -1.0, C, ldc)
        want = C.copy()
        assert oracle.gemm_work("T", "N", 200, 131, 300, 2.0, A, lda, B, ldb, -1.0, want, ldc) == 0
        assert np.array_equal(out, want, equal_nan=True)
        for uplo, trans in itertools.product("LU", "NT"):
            A, lda, C, ldc = make_syrk_operands(rng, trans, 203, 45, (1, 1), dtype)
            assert check_syrk_full(xg, uplo, trans, 203, 45, 1.5, A, lda, -0.5, C, ldc) < 1.0
            assert "64x64" in xg.xgemm_last_kernel_name() or "32x32" in xg.xgemm_last_kernel_name()
    print("fallback ok", flush=True)


if __name__ == "__main__":
    main()
