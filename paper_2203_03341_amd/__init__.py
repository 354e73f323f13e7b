"""Error-corrected SGEMM for MI355X: thin Python face of the C-ABI library (see include/ecgemm.h)."""
from .binding import (ERR_ALLOC, ERR_HIP, ERR_INVALID_ARG, ERR_UNSUPPORTED, MODE_BF16_FULL, MODE_BF16_PLAIN, MODE_FP16_MARKIDIS, MODE_FP16_OUTSIDE_ACC, MODE_FP16_OUTSIDE_ACC_4, MODE_FP16_OUTSIDE_ACC_16, MODE_AUTO,
                      MODE_FP16_PLAIN, MODE_FP16_SPLIT, MODE_FP16_UNSCALED, MODE_FP32_MFMA, OK, OP_N, OP_T, SHAPE_32x32_FUSED, SHAPE_64x64_FUSED, SHAPE_128x128_X2, SHAPE_256x128_W4,
                      SHAPE_AUTO, NOALLOC_WORKSPACE_BYTES, EcgemmError, Handle, debug_tile_order, plan_info, split_size,
                      status_string, workspace_size)

__all__ = ["Handle", "EcgemmError", "split_size", "workspace_size", "plan_info", "debug_tile_order", "status_string", "OP_N", "OP_T", "MODE_FP16_SPLIT", "MODE_BF16_FULL", "MODE_FP16_MARKIDIS", "MODE_FP16_UNSCALED", "MODE_FP16_PLAIN", "MODE_BF16_PLAIN", "MODE_FP16_OUTSIDE_ACC", "MODE_FP16_OUTSIDE_ACC_4", "MODE_FP16_OUTSIDE_ACC_16", "MODE_AUTO", "MODE_FP32_MFMA",
           "SHAPE_AUTO", "SHAPE_256x128_W4", "SHAPE_128x128_X2", "SHAPE_64x64_FUSED", "SHAPE_32x32_FUSED",
           "NOALLOC_WORKSPACE_BYTES", "OK", "ERR_INVALID_ARG", "ERR_ALLOC", "ERR_HIP", "ERR_UNSUPPORTED"]
