"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

Holds no arithmetic of the method (no binarisation, packing, products or
activations): only counter-based random tensors and the shapes of the five
benchmark configurations.
"""
from .synth import (  # noqa: F401
    NetConfig, GemmShape, CONFIGS, GEMM_SWEEP, get_config,
    uniform_pm1, normal, random_words, make_net_params, make_frames,
    TENSOR_W, TENSOR_BIAS, TENSOR_INPUT, TENSOR_ABITS, TENSOR_BBITS,
)
