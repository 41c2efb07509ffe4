"""MI355X-native binary-codebook linear layer (btc_pack / btc_gemv / btc_gemm).

The product is the C-ABI library built from csrc/ (declared in include/btc.h);
this package holds its in-tree build step and a thin ctypes binding.
"""
from .binding import (  # noqa: F401
    BTC_BF16, BTC_F16, BTC_F32, BTC_OK, BtcError, btc_aq_workspace_bytes, btc_assign, btc_gemm, btc_gemm_aq, btc_gemv, btc_gemv_engine, btc_gemv_groups, btc_gemv_multi, btc_gemv_multi_shapes, btc_gemv_static, btc_gemv_transformed, btc_gemv_transformed_multi, btc_gemv_transformed_workspace_bytes, btc_pack, btc_packed_bytes, btc_quantize_rows, btc_shape,
    btc_shape_init, btc_transform, btc_transform_prepare, btc_transform_prepared_bytes, btc_unpack, btc_update, btc_update_workspace_bytes, btc_weight_rowsums, btc_workspace_bytes, lib, status_str,
)
