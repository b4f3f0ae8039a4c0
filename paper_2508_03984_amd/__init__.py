"""oz2: DGEMM / SGEMM emulation on MI355X INT8 matrix cores (Ozaki scheme II).

The work is done by liboz2.so (hand-written HIP for gfx950, C ABI in
include/oz2.h).  This package is the thin binding: the functions of
`paper_2508_03984_amd.binding` carry the same names as the C entry points and
only marshal arguments; torch supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    OZ2Error, lib_path, load, oz2_constants, oz2_dgemm, oz2_dgemm_accurate, oz2_int8_gemm,
    oz2_sgemm_accurate, oz2_shift_table_accurate, oz2_mfma_probe,
    oz2_last_stage_times_ms, oz2_release, oz2_set_int32_products, oz2_set_profiling, oz2_set_workspace,
    oz2_sgemm, oz2_shift_table, oz2_stage_ptr, oz2_status_string, oz2_workspace_bytes,
    stage_tensor, matmul, block_slices, unblock_slices,
    OZ2_OP_N, OZ2_OP_T, Operand, oz2_dgemm_op, oz2_sgemm_op, oz2_prepare_d, oz2_prepare_s, oz2_operand_free,
    oz2_operand_bytes, oz2_dgemm_prepared, oz2_sgemm_prepared, oz2_workspace_min_bytes,
    oz2_set_workspace_limit, oz2_last_panels, oz2_plan_panels, oz2_set_overlap, oz2_set_small_conversion,
    oz2_dgemm_colmajor, oz2_sgemm_colmajor,
)
