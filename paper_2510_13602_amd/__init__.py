"""NOSA decode-step hot path for AMD MI355X (gfx950): hand-written HIP kernels behind a C ABI.

``include/nosa.h`` declares the library; ``binding`` marshals PyTorch tensors into it.
"""
from .binding import (DTYPE_BF16, DTYPE_F32, EXPORTS, KERNEL_APPEND, KERNEL_COMBINE, KERNEL_DECODE,  # noqa: F401
                      KERNEL_EVICT, KERNEL_FETCH, KERNEL_NAMES, KERNEL_PREFILL,
                      KERNEL_SCORE, KERNEL_SELECT, LIB_PATH, MAX_SPLITS, Nosa, NosaError, Params, STATIC_SCRATCH_BYTES, StepArgs,
                      load_library, make_params, validate_params)
