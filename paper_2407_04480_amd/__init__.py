"""MI355X-native implementation of LoCo's per-step local path (arXiv 2407.04480, Alg. 1).

`binding` wraps the C-ABI library (include/loco.h) built from csrc/*.hip;
`workloads` makes the seeded synthetic gradients; `build` compiles the library.
Importing the package loads nothing: the library is opened on first use and a
missing library is an error, never a fallback.
"""
from .binding import (  # noqa: F401
    LocoError,
    library_path,
    loco_code_bytes,
    loco_num_blocks,
    loco_error_state_init,
    loco_compensate_quantize,
    loco_dequant_reduce,
    loco_reset_due,
    loco_error_state8_init,
    loco_compensate_quantize_fixed,
    loco_dequant_reduce_fixed,
    loco_compensate_quantize_clip,
    loco_compensate_quantize_fixed_clip,
    loco_dequant_reduce_sgd,
    loco_dequant_reduce_adam,
    loco_dequant_reduce_fixed_sgd,
    loco_dequant_reduce_fixed_adam,
    loco_dequant_reduce_bf16,
    loco_dequant_reduce_fixed_bf16,
    loco_compensate_quantize_bf16_scales,
    loco_dequant_reduce_bf16_scales,
    loco_stream_copy,
    loco_stream_read,
    loco_stream_fill,
    loco_stream_sum2,
    loco_device_info,
)

__all__ = [
    "LocoError",
    "library_path",
    "loco_code_bytes",
    "loco_num_blocks",
    "loco_error_state_init",
    "loco_compensate_quantize",
    "loco_dequant_reduce",
    "loco_reset_due",
    "loco_error_state8_init",
    "loco_compensate_quantize_fixed",
    "loco_dequant_reduce_fixed",
    "loco_compensate_quantize_clip",
    "loco_compensate_quantize_fixed_clip",
    "loco_dequant_reduce_sgd",
    "loco_dequant_reduce_adam",
    "loco_dequant_reduce_fixed_sgd",
    "loco_dequant_reduce_fixed_adam",
    "loco_dequant_reduce_bf16",
    "loco_dequant_reduce_fixed_bf16",
    "loco_compensate_quantize_bf16_scales",
    "loco_dequant_reduce_bf16_scales",
    "loco_stream_copy",
    "loco_stream_read",
    "loco_stream_fill",
    "loco_stream_sum2",
    "loco_device_info",
]
