"""Python binding of libbsr_spmm: the block-sparse product Y = X * W^T on MI355X.

Argument marshalling only: every step of the product runs in the HIP kernels of the C-ABI
library declared in include/bsr_spmm.h.  PyTorch supplies device memory and the stream.
There is no CPU fallback: if the library is not built, importing the entry points raises.
"""
from .binding import (BsrMatrix, BsrError, PATH_AUTO, PATH_MFMA, PATH_WAVE, bsr_create, bsr_create_transposed, bsr_transpose_pattern, bsr_query_path,
                      bsr_scratch_size, bsr_spmm, bsr_spmm_ex, bsr_spmm_static, STATIC_SCRATCH_BYTES, bsr_sddmm, bsr_tune, bsr_tune_result, bsr_status_string, bsr_validate, bsr_workspace_size,
                      library_path, load_library)

__all__ = ["BsrMatrix", "BsrError", "PATH_AUTO", "PATH_MFMA", "PATH_WAVE", "bsr_create", "bsr_create_transposed", "bsr_transpose_pattern", "bsr_query_path",
           "bsr_scratch_size", "bsr_spmm", "bsr_spmm_ex", "bsr_spmm_static", "STATIC_SCRATCH_BYTES", "bsr_sddmm", "bsr_tune", "bsr_tune_result", "bsr_status_string", "bsr_validate", "bsr_workspace_size",
           "library_path", "load_library"]
