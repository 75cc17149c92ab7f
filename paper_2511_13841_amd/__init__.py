"""MI355X (gfx950) batched speculative-verification library: Python binding.

The binding only marshals arguments to the C ABI of libdas.so (include/das.h);
every step of the path runs in the library's HIP kernels.
"""
from .binding import (DasModel, DasError, lib, config_for, debug_gemm, debug_gemm_silu, debug_gemm_rowmax, debug_gemm_time, gemm_noalloc, debug_copy, debug_copy_ring, debug_mfma_loop, kernel_classes,
                      DAS_OK, DAS_ERR_INVALID, DAS_ERR_STATE, DAS_ERR_NOMEM, DAS_ERR_DEVICE)
