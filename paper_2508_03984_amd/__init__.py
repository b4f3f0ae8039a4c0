"""oz2: DGEMM / SGEMM emulation on MI355X INT8 matrix cores (Ozaki scheme II).

The work is done by liboz2.so (hand-written HIP for gfx950, C ABI in
include/oz2.h).  This package is the thin binding: the functions of
`paper_2508_03984_amd.binding` carry the same names as the C entry points and
only marshal arguments; torch supplies device memory and streams.
"""
from . import binding as _binding
from .binding import (  # noqa: F401
    OZ2Error, lib_path, load, stage_tensor, matmul, block_slices, unblock_slices, OZ2_OP_N, OZ2_OP_T, Operand, Context,
    OZ2_OPT_INT32_PRODUCTS, OZ2_OPT_OVERLAP, OZ2_OPT_SMALL_CONVERSION, OZ2_OPT_PROFILING,
)

# one Python function per C entry point, under the same name
globals().update({_name: getattr(_binding, _name) for _name in _binding.EXPORTS})
