"""MI355X-native convolution library (Winograd F(n,k) / 1x1 GEMM / direct + planner).

Thin ctypes binding over libmnnconv.so; every step of the path runs in the HIP
kernels behind the C ABI declared in include/mnn_conv.h.
"""
from .binding import (  # noqa: F401
    ConvPlan, MnnError, Scheme, Options, lib, library_path,
    get_transforms, analytic_cost, analytic_tile, enumerate_schemes, select_scheme,
    cache_size, cache_clear, version,
    SCHEME_AUTO, SCHEME_DIRECT, SCHEME_WINOGRAD, SCHEME_GEMM1X1, GEMM_FP32, GEMM_BF16,
    STAGE_FILTER, STAGE_INPUT, STAGE_GEMM, STAGE_OUTPUT, STAGE_COUNT, BUF_U, BUF_V, BUF_M,
)
