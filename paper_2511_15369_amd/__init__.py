"""MI355X-native integer softmax / GELU / requantization of IPTQ-ViT (arXiv 2511.15369).

Thin Python binding over the C-ABI library ``libiptq.so`` (hand-written HIP kernels for
gfx950).  PyTorch is used only for device memory and streams.
"""

from .binding import (  # noqa: F401
    ALGO_AUTO,
    ALGO_DYNAMIC,
    ALGO_GENERIC,
    ALGO_SLAB,
    ALGO_WIDE,
    BATCH_MAX,
    Dyadic,
    GeluProblem,
    SoftmaxProblem,
    GeluParams,
    IptqError,
    SoftmaxParams,
    gelu_i8,
    gelu_i8_batch,
    gelu_i8_layers,
    gelu_problem,
    gelu_i32,
    gelu_prepare,
    lib_path,
    load,
    make_dyadic,
    requant,
    softmax_i32,
    softmax_i32_batch,
    softmax_i32_layers,
    softmax_kernel_family,
    softmax_problem,
    softmax_prepare,
    strerror,
    version,
)
