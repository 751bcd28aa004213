"""MI355X-native GEMM (dgemm / sgemm / split-plane zgemm) behind a C ABI.

The compute lives in ``libxgemm.so`` (hand-written HIP for gfx950, built by
``python -m paper_1611_08035_amd.build``).  This package is only the thin
binding: argument marshalling from torch tensors (device memory, streams) to
the C entry points declared in ``include/xgemm.h``.  There is no CPU fallback:
if the library is missing, every call raises.
"""
from .xgemm import (  # noqa: F401
    XgemmError,
    lib,
    library_path,
    xgemm_dgemm,
    xgemm_sgemm,
    xgemm_dsyrk,
    xgemm_ssyrk,
    xgemm_dtrsm,
    xgemm_strsm,
    xgemm_dtrmm,
    xgemm_strmm,
    xgemm_dsyr2k,
    xgemm_ssyr2k,
    xgemm_dsymm,
    xgemm_ssymm,
    xgemm_dpotrf,
    xgemm_spotrf,
    xgemm_tile_map,
    xgemm_workspace_bytes,
    xgemm_workspace_init,
    xgemm_dgemm_ws,
    xgemm_sgemm_ws,
    xgemm_dsyrk_ws,
    xgemm_ssyrk_ws,
    xgemm_force_split,
    xgemm_last_split,
    xgemm_plan,
    xgemm_zgemm_split,
    xgemm_zgemm,
    xgemm_zgemm_workbytes,
    xgemm_zgemm_worksize,
    xgemm_version,
    xgemm_last_kernel_name,
    xgemm_force_variant,
    xgemm_variant_name,
    xgemm_mfma_peak_probe,
    xgemm_mfma_layout_probe,
    xgemm_hwid_probe,
    xgemm_latency_probe,
    xgemm_model_outer_product_rate,
    xgemm_model_stalled_rate,
    xgemm_model_n_updates,
    xgemm_model_predict,
    EXPORTS,
)
