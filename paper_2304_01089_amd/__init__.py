"""MI355X (gfx950) implementation of the RPTQ inference hot path.

The product is the C-ABI library `librptq.so` (see include/rptq.h); this package is its
thin Python binding: same entry-point names, argument marshalling only.  PyTorch supplies
device memory and streams.  There is no CPU fallback: calling any entry point without the
built library raises.
"""
from .binding import (  # noqa: F401
    RptqError,
    library_path,
    load_library,
    rptq_padded_k,
    rptq_codes_bytes,
    rptq_weight_bytes,
    rptq_calibrate_workspace_bytes,
    rptq_cluster_channels,
    rptq_channel_minmax,
    rptq_calibrate,
    rptq_fold_reorder,
    rptq_ln_quant,
    rptq_ln_quant_scatter,
    rptq_ln_quant_scatter_workspace_bytes,
    rptq_cluster_gemm,
    rptq_cluster_gemm_quant,
    rptq_cluster_gemm_quant_workspace_bytes,
    rptq_cluster_gemm_quant_static,
    rptq_cluster_gemm_partials,
    rptq_unpack_codes,
    rptq_unpack_weights,
    rptq_cw_scale_bytes,
    rptq_cw_cross_bytes,
    rptq_cw_rowsum_bytes,
    rptq_fold_reorder_cw,
    rptq_cluster_rowsums,
    rptq_cluster_gemm_cw,
    rptq_cluster_gemm_partials_cw,
    rptq_cluster_heads,
    rptq_kv_table_bytes,
    rptq_kv_tables,
    rptq_kv_quant,
    rptq_kv_dequant,
    rptq_dequant_codes,
    rptq_dequant_weights,
    rptq_gemm_bf16,
    rptq_device_info,
    rptq_strerror,
    rptq_version,
    EXPORTED_SYMBOLS,
    DTYPE_BF16,
    DTYPE_F32,
)
from .layer import (Calibration, FoldedLinear, FoldedLinearCw, calibrate_site, identity_site, fold_linear, ln_quant,  # noqa: F401
                    cluster_gemm, cluster_gemm_quant, fold_linear_cw, cluster_rowsums, cluster_gemm_cw)
