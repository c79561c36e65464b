"""MI355X-native PTQTP decode hot path: thin ctypes binding over libptqtp.so.

Argument marshalling only -- every step of the path runs in the HIP kernels of
csrc/*.hip.  PyTorch is used for device memory and streams.  There is no
CPU fallback: importing the binding fails loudly when the library is missing.
"""
from .binding import (  # noqa: F401
    PTQTP_F16, PTQTP_F32, PTQTP_FUSED_PLANES, PTQTP_GEMM_SMALL_MAX_M, PtqtpError, lib_path,
    BatchPlan, ptqtp_gemm, ptqtp_gemm_batch, ptqtp_gemm_batch_fused, ptqtp_gemm_small, ptqtp_gemv, ptqtp_gemv_batch, ptqtp_gemv_batch_plan, ptqtp_pack, ptqtp_check_blob, ptqtp_quantize, ptqtp_quantize_static, PTQTP_QUANTIZE_STATIC_BYTES, ptqtp_packed_bytes, ptqtp_status_string,
    ptqtp_tune, ptqtp_unpack, ptqtp_version, ptqtp_workspace_bytes, ptqtp_gemm_route,
    PTQTP_ROUTE_STREAM, PTQTP_ROUTE_SMALL, PTQTP_ROUTE_SMALL_CHUNKS, PTQTP_ROUTE_TILE, TILE_SHAPES,
    PTQTP_BLOB_BAD_MAGIC, PTQTP_BLOB_BAD_LAYOUT, PTQTP_BLOB_BAD_GROUP, PTQTP_BLOB_BAD_N, PTQTP_BLOB_BAD_K,
    PTQTP_EPI_NONE, PTQTP_EPI_SWIGLU, ChainPlan, ptqtp_chain_plan, ptqtp_chain_run, ptqtp_chain_run_batch,
)
