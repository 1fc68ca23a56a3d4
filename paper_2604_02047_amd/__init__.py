"""MI355X-native tree verification for anisotropic spine-tree speculative decoding.

The work is done by libgoose.so (hand-written HIP for gfx950, C ABI in include/goose.h).
This package is a thin ctypes binding with the same entry-point names; PyTorch only
provides device memory and streams.
"""
from .binding import (  # noqa: F401
    GooseError,
    GooseContext,
    ModelDesc,
    goose_check_parent,
    goose_packed_matrix_bytes,
    goose_pack_matrix,
    goose_gemm_packed,
    goose_gemm_swiglu_packed,
    goose_gemm_packed_ex,
    goose_gemm_swiglu_packed_ex,
    goose_split_operand,
    goose_lm_head_argmax_static,
    lib_path,
    load_library,
    EXPORTS,
)
