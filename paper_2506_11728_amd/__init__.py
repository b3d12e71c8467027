"""MI355X-native mixed-precision integer GEMM (int8 x int8 -> int32): Python binding of libmipgemm."""
from .binding import (  # noqa: F401
    ROW_MAJOR, COL_MAJOR, OVERWRITE, ACCUMULATE, MipGemmError,
    library_path, load_library, exported_symbols,
    mipgemm_s8s8s32, mipgemm_u8s8s32, mipgemm_s8u8s32,
    mipgemm_s8s8s32_batched, mipgemm_u8s8s32_batched, mipgemm_s8u8s32_batched,
    mipgemm_s8s8f32, mipgemm_u8s8f32, mipgemm_s8u8f32,
    mipgemm_s8s8s8, mipgemm_u8s8s8, mipgemm_s8u8s8,
    mipgemm_workspace_size, mipgemm_workspace_size_f32, mipgemm_strerror, mipgemm_variant_name,
    mipgemm_variant_name_with_workspace, mipgemm_variant_name_for_mode, mipgemm_mfma_ceiling,
    mipgemm_set_tuning, tuning, mipgemm_s8s8s32_noalloc, mipgemm_static_scratch_bytes, ERR_STATIC_SCRATCH, mipgemm_mfma_ceiling_clocked, mipgemm_s8s8s32_clocked, mipgemm_conv_workspace_size_unaligned,
    mipgemm_conv_s8u8s32, mipgemm_conv_s8u8f32, mipgemm_conv_workspace_size, mipgemm_conv_variant_name, mipgemm_im2col_u8, mipgemm_pack_b,
    mipgemm_packed_weights_bytes, mipgemm_pack_weights, mipgemm_s8s8s32_packed, mipgemm_u8s8s32_packed,
    mipgemm_conv_filter_sums, mipgemm_conv_s8u8s32_with_sums, mipgemm_conv_s8u8f32_with_sums, mipgemm_conv_s8u8s8,
    mipgemm_s16s16s32, mipgemm_workspace_size_s16,
)
