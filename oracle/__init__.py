"""CPU oracle for the MIP GEMM (test infrastructure, never part of the product path)."""
from .mip_oracle import (  # noqa: F401
    ROW_MAJOR, COL_MAJOR, OVERWRITE, ACCUMULATE,
    build, gemm, gemm_s16, gemm_dequant, gemm_requant, gemm_s8s8s32, gemm_u8s8s32, gemm_s8u8s32, num_threads,
    conv_direct, conv_out_extent, im2col_u8, pack_b, column_sums, pack_weights, packed_weights_layout,
)
