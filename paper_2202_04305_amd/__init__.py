"""spmi: sparse x dense products under per-level dense/compressed storage on MI355X.

Thin binding over the C ABI in include/spmi.h.  Everything computed runs in the HIP
library; Python only marshals arguments.  PyTorch supplies device memory and the stream.
"""
from .binding import (  # noqa: F401
    SpError, Encoding, Tensor, sp_encode, sp_pack, sp_prepare, sp_matmul, sp_matmul_noalloc, sp_pos, sp_crd, sp_values, sp_unpack, sp_convert, sp_sddmm, sp_mttkrp, sp_spgemm, sp_add,
    sp_tensor_info, sp_tensor_tune, sp_profile_read, sp_stream_copy, sp_stream_read, sp_pack_sort_mode, load_library,
    SP_DENSE, SP_COMPRESSED, SP_F32, SP_F64, SP_TUNE_SPMV_KERNEL, SP_TUNE_CSC_MODE, SP_TUNE_SPMM_KERNEL, SP_TUNE_PROFILE, SP_TUNE_SPGEMM_KERNEL,
)
