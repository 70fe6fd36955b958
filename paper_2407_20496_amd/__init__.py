"""HiNM sparse GEMM with fused channel permutation for AMD MI355X (gfx950).

Thin binding over the C ABI in ``include/hinm.h`` (``libhinm.so``): argument
marshalling only -- every step of the path runs in the HIP kernels.  PyTorch is
used for device memory and streams.  There is no CPU fallback: if the shared
library is missing, every call raises.

16-bit tensors may be passed as ``torch.float16`` / ``torch.bfloat16`` or as
``torch.int16``/``torch.uint16`` bit patterns together with ``dtype="f16"|"bf16"``.
"""
from __future__ import annotations

from .binding import (  # noqa: F401
    F16, BF16, EPI_RELU, OUT_F32, KERNEL_REFERENCE, KERNEL_SMFMAC, KERNEL_GEMV,
    HinmError, Layer, library_path, load_library, exported_symbols,
    hinm_pack_sizes, hinm_pack, hinm_pack_static, PACK_STATIC_MAX_SCORES, hinm_pack_ordered, hinm_tile_order, hinm_apply_row_order, hinm_pack_scored, hinm_pack_vectors, hinm_unpack, hinm_spmm,
    hinm_spmm_vectors, hinm_icp_sizes, hinm_icp_search, hinm_ocp_sizes, hinm_ocp_search, hinm_ocp_cluster_sizes, hinm_ocp_cluster,
    hinm_chain_sizes, hinm_chain,
    hinm_prepare_sizes, hinm_prepare, hinm_spmm_prepared_workspace, hinm_spmm_prepared, hinm_spmm_prepared_plan,
    hinm_status_str, hinm_version,
    calib_symbols, hinm_calib_copy, hinm_calib_fill, hinm_calib_read, hinm_calib_scatter_rows, hinm_calib_smfmac,
    hinm_calib_empty, hinm_calib_lds_stream, hinm_calib_gather_stream, hinm_calib_tile_part,
)
