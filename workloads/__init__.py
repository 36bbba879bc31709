"""Seeded synthetic inputs shaped like the ViT / DeiT / Swin workloads.

This package only draws random tensors and real-valued scales.  It contains none
of the integer softmax / GELU / requantization arithmetic, so both the CPU
oracle's tests and the HIP path's tests and benchmark can take inputs from it
without sharing any part of the method.
"""

from .generators import (  # noqa: F401
    CONFIGS,
    SoftmaxCase,
    GeluCase,
    config_names,
    gelu_case,
    gelu_input,
    layer_scales,
    qk_pair,
    scores_from_qk,
    softmax_bias,
    softmax_case,
    softmax_qk,
    swin_bias,
    detection_key_mask,
    shifted_window_mask,
    SWIN_B_MAP_SIDE,
)
