"""MI355X-native quantized GNN layer (QGTC, arXiv 2111.09547): Python binding
of the C-ABI library libqgtc.so.  PyTorch is used for device memory and streams
only; every step of the path runs in the library's HIP kernels."""
from .binding import (  # noqa: F401
    LEFT, RIGHT, RIGHT_BYTES, LEFT_BYTES, OUT_I32, OUT_F32, OUT_BITS,
    KERNEL_PACK, KERNEL_TILE_MAP, KERNEL_AGGREGATE, KERNEL_UPDATE, KERNEL_SUMS, KERNEL_LAYER,
    QgtcError, Bits, TileMap, Epilogue, lib, lib_path, describe, alloc_bits,
    qgtc_pack_bits, qgtc_unpack_bits, qgtc_build_tile_map, qgtc_aggregate,
    qgtc_update, qgtc_layer, qgtc_layer_static, LAYER_STATIC_MAX_BYTES, qgtc_row_sums, qgtc_col_sums,
    Tuning, LAYER_FUSED, LAYER_TWO_KERNELS, UPDATE_AUTO, UPDATE_POPCOUNT, UPDATE_MATRIX_CORES,
    ZERO_WORDS_AUTO, ZERO_WORDS_VISIT, ZERO_WORDS_SKIP,
    qgtc_tile_stats, tile_stats_numbers, qgtc_plan_layer, qgtc_quant_inv_scale, qgtc_layer_epilogues, qgtc_fold_batchnorm, qgtc_device_info,
    qgtc_probe_popcount, qgtc_prof_enable, qgtc_prof_reset, qgtc_prof_read, qgtc_version,
)
