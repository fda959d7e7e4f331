"""MI355X-native fp32 GEMM (C = A.B, single and batched) behind a C-ABI library.

``binding`` marshals torch device tensors into ``libtgemm.so``; every arithmetic step
runs in the HIP kernels.  ``inputgen`` holds the seeded synthetic operands (numpy only).
Nothing is loaded at import time; the shared library is opened on first use and its
absence is an error (there is no fallback path).
"""
from .binding import (  # noqa: F401
    MATH_BF16_PIECES,
    MATH_FP32_MFMA,
    TgemmError,
    clear_tune_cache,
    force_config,
    candidates,
    get_config,
    get_math,
    set_math,
    kernel_names,
    last_config,
    library_path,
    load_library,
    open_library,
    poison_library_path,
    load_tune_cache,
    save_tune_cache,
    saxpy,
    set_workspace,
    sgemm,
    sgemm_batched,
    sgemm_splitk_static,
    sgemm_strided,
    tune,
    tune_is_launch_bound,
    version,
    workspace_bytes,
    strided_workspace_bytes,
)
