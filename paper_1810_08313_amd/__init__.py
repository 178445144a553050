"""MI355X-native local-update SGD (PASGD) with the AdaComm controller.

The package is a thin binding over liblocalcomm.so (C ABI in
include/localcomm.h, HIP sources in csrc/).  Nothing here computes on the CPU.
"""
from .binding import (  # noqa: F401
    GEMM_BF16,
    GEMM_FP32,
    KIND_MLP,
    KIND_QUAD,
    LcError,
    LcModel,
    LocalSGD,
    adacomm_next_tau,
    adacomm_next_tau_ex, average_block_momentum_static, STATIC_MAX_PARAMS,
    lc_param_count,
    lc_row_stride,
    lib,
    make_model,
)
