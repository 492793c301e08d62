"""MI355X (gfx950) library for the data-parallel hot path of Global-QSGD (arXiv 2305.18627).

The product is the C-ABI shared library built from csrc/ (see include/gqsgd.h); this package is
its ctypes binding with the same call names.
"""
from .binding import (  # noqa: F401
    GQ_AGG_I16, GQ_AGG_I32, GQ_ERR_DEVICE, GQ_FLAG_WRITE_WINDOWS_OFF, GQ_FLAG_WRITE_WINDOWS_ON, GQ_ERR_INVALID_ARG, GQ_ERR_OVERFLOW, GQ_ERR_UNSUPPORTED,
    GQ_ERR_WORKSPACE, GQ_EXP, GQ_LINEAR, GQ_MAX_WORKERS, GQ_NORM_L2, GQ_NORM_L2_MAX, GQ_NORM_LINF, GQ_OK,
    GQ_PACK_I4, GQ_PACK_I8, GQ_PACK_U4_SIGNPLANE, GQ_PACK_U8_SIGNPLANE, GQError, avg_reduce, bucketed_quantize_aggregate, bucketed_workspace_bytes, check_width, compact, compact_workspace_bytes, dequantize, exp_reduce, sparse_aggregate,
    fused_quantize_aggregate, global_norm, global_norm_static, gq_params, int_aggregate, levels_nbytes, lib, make_params,
    norm_workspace_bytes, quantize, quantize_compact, signplane_nwords, sparse_nnz_bound, status_string, tile_starts_len, version,
)
