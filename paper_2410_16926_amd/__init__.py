"""MI355X-native group-wise Pyramid Vector Quantization (encode / decode / decode fused into a
matrix-vector product) behind the C library declared in include/pvq.h."""
from .binding import (  # noqa: F401
    PVQ_BF16, PVQ_F16, PVQ_F32, DIAGNOSTICS, EXPORTS, Packed, PvqContext, PvqError, alloc_packed, lib,
    pvq_beta_tables, pvq_count, pvq_ctx_create, pvq_ctx_destroy, pvq_ctx_set_amplitude, pvq_decode, pvq_decode_gemv,
    pvq_encode, pvq_fast_tables_selftest, pvq_walk_tables_selftest, pvq_max_k, pvq_packed_sizes, pvq_size_table_device, pvq_hadamard, pvq_rotate_encode, pvq_correct,
    pvq_correct_static, pvq_correct_static_max_rows, pvq_correct_set_front_tiles, pvq_decode_set_table_decoder_min_groups, pvq_decode_gemv_plan,
)
