"""MI355X-native PTQ4VM quantized-linear path (arXiv 2412.20386).

`binding` exposes the C ABI of libptq4vm.so (hand-written HIP for gfx950); `synth` draws the
seeded Vim-shaped inputs; `build` compiles the library.  Nothing is loaded at import time.
"""
from . import binding, synth  # noqa: F401
from .binding import (  # noqa: F401
    Ptq4vmError,
    f16_linear,
    fold_smoothing,
    fold_smoothing_w4,
    quantize_pts_a4,
    w4a4_linear,
    e2m3_blocks,
    fold_smoothing_w4_e2m3,
    quantize_pts_a4_e2m3,
    w4a4_linear_e2m3,
    w4a4_linear_fused,
    quantize_dynamic,
    quantize_pts,
    quantize_pts_offset,
    weight_rowsum,
    w8a8_linear_offset,
    w8a8_linear_offset_fused,
    w8a8_linear,
    w8a8_linear_fused,
    validate_scales,
    validate_scales_static,
)
