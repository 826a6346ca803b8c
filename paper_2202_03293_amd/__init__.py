"""liblg: the paper's dense structured tensor ops (matmul, conv2d, depthwise conv, row/column
reductions, transpose, copy) as hand-written HIP kernels for one MI355X, behind a C ABI.

The Python layer only marshals arguments: every function below passes device pointers, extents
and the current HIP stream to the C entry point of the same name in liblg.so.  There is no
fallback: importing the ops without the built library raises.
"""
from .ops import (  # noqa: F401
    LgError, lib, lg_version, lg_status_string, lg_conv_out_extent,
    lg_matmul, lg_matmul_t, lg_matmul_workspace_bytes, lg_matmul_plan, lg_matmul_t_plan,
    lg_matmul_plan_tile_loop, lg_gemm_variants, lg_gemm_variant_info, lg_gemm_variant_workspace_bytes, lg_matmul_variant,
    lg_conv2d_nhwc_hwcf_variant,
    lg_conv2d_nhwc_hwcf, lg_conv2d_workspace_bytes, lg_conv1d_nwc_wcf, lg_conv1d_workspace_bytes,
    lg_dwconv1d_nwc_wc, lg_dwconv2d_nhwc_hwc,
    lg_reduce_rows, lg_reduce_rows_ws, lg_reduce_rows_workspace_bytes, lg_reduce_cols, lg_reduce_cols_workspace_bytes,
    lg_reduce_cols_static,
    lg_transpose, lg_transpose_batched, lg_copy2d,
    lg_mfma_probe, lg_mfma_probe_out_elems, lg_mfma_probe_flops, lg_stream_probe,
)
