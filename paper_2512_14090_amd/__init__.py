"""MI355X-native scheme scoring for Arithmetic-Intensity-Aware Quantization.

Thin Python binding over libaiq.so (hand-written HIP kernels for gfx950 behind a
C boundary, declared in include/aiq.h).  The binding marshals arguments only;
PyTorch supplies device memory and streams.  There is no CPU fallback: without
the built library, or without a GPU, the device entry points raise.
"""
from .binding import (  # noqa: F401
    AiqError, Model, Deployed, layer_ai, quantize_weights, library_path, load_library, EXPORTED_SYMBOLS,
    K_QUANTIZE, K_CONV, K_DEPTHWISE, K_HEAD, K_AGREE, K_FUSED, K_MBCONV, K_CONV_CODES, MODEL_LAYERWISE, MODEL_PER_TENSOR, MODEL_ACT_QUANT,
    DEPLOY_FP32_MATRIX,
)
