"""MI355X-native LeanQuant per-layer quantization pass (C-ABI library + thin binding)."""
from .binding import (  # noqa: F401
    LQ_CALL_CHOLESKY, LQ_CALL_EXACT, LQ_CALL_FIT_GRID, LQ_CALL_HESSIAN, LQ_CALL_QUANTIZE, LQ_ERR_HIP,
    LQ_ERR_INVALID_ARG, LQ_ERR_NOT_PD, LQ_ERR_UNSUPPORTED, LQ_ERR_WORKSPACE, LQ_GRID_AFFINE,
    LQ_GRID_NONUNIFORM, LQ_OK, LeanQuantError, alloc_workspace, grid_shape, load, params_for, lq_bits_per_weight,
    lq_cholesky_inv, lq_fit_grid, lq_fit_grid_from, lq_fit_grid_static, lq_hessian_accumulate, lq_hessian_accumulate_host,
    lq_hessian_host_workspace_bytes, lq_last_error, lq_matmul_packed, lq_matvec_packed, lq_pack_layer, lq_packed_row_bytes,
    lq_hinv_from_factor, lq_kmeanspp_seed, lq_params, lq_params_default, lq_quantize_exact, lq_quantize_layer, lq_unpack_layer, lq_version,
    lq_workspace_bytes)
