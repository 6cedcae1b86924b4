"""Tile-wise / tile-vector-wise sparse GEMM for MI355X: thin Python binding
over the C-ABI library libtwgemm.so (see include/twgemm.h)."""
from .binding import (  # noqa: F401
    TwError, PackedWeight, lib, lib_path, tw_pack, tw_pack_host, tw_pack_dev, tw_prune_dev, tw_prune_workspace_bytes, tw_prune_dev_static, tw_concat, tw_gemm,
    tw_dense_gemm, tw_pack_i8, tw_pack_i8_host, tw_gemm_i8, tw_dense_gemm_i8, tw_conv_bind, tw_conv_gemm, tw_conv_gemm_i8, ConvBinding, LaunchOpts, tw_launch_opts, tw_gemm_ex, tw_gemm_workspace_bytes, tw_workspace_init, DTYPE_F16, DTYPE_I8,
    tw_set_option, tw_calibrate, CAL_COPY, CAL_READ, CAL_WRITE, CAL_STORE_CT, CAL_MFMA_F16, CAL_SMFMAC_F16, CAL_MFMA_I8, PATTERN_TW, PATTERN_TVW, PATTERN_TEW, LAYOUT_KM, LAYOUT_MK, EXPORTED_SYMBOLS,
)
