"""ctypes binding of the C-ABI library (include/loco.h): argument marshalling only.

The functions carry the names of the C entry points.  Tensors are torch tensors
on the GPU (torch is used for device memory and streams only); every step of the
method runs in the library's HIP kernels.  There is no CPU path: a missing
library, a CPU tensor or a non-zero status raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libloco.so")

LOCO_OK = 0
LOCO_F32 = 0
LOCO_BF16 = 1

EXPORTS = (
    "loco_status_string",
    "loco_code_bytes",
    "loco_num_blocks",
    "loco_set_pointer_checks",
    "loco_error_state_init",
    "loco_compensate_quantize",
    "loco_dequant_reduce",
    "loco_compensate_quantize_bf16_scales",
    "loco_dequant_reduce_bf16_scales",
    "loco_stream_copy",
    "loco_stream_read",
    "loco_stream_fill",
    "loco_stream_sum2",
    "loco_device_info",
    "loco_reset_due",
    "loco_error_state8_init",
    "loco_compensate_quantize_fixed",
    "loco_compensate_quantize_fixed_f32state",
    "loco_dequant_reduce_fixed",
    "loco_compensate_quantize_clip",
    "loco_compensate_quantize_fixed_clip",
    "loco_dequant_reduce_sgd",
    "loco_dequant_reduce_adam",
    "loco_dequant_reduce_fixed_sgd",
    "loco_dequant_reduce_fixed_adam",
    "loco_dequant_reduce_bf16",
    "loco_dequant_reduce_fixed_bf16",
    "loco_compensate_quantize_scheduled",
    "loco_compensate_quantize_fixed_scheduled",
    "loco_compensate_quantize_fixed_f32state_scheduled",
    "loco_step_index_set",
    "loco_step_index_advance",
    "loco_dequant_reduce_decomposed",
    "loco_dequant_reduce_decomposition",
    "loco_runtime_copy",
    "loco_stream_update3",
    "loco_compensate_quantize_staged_codes",
    "loco_compensate_quantize_resident",
)

_lib = None


class LocoError(RuntimeError):
    def __init__(self, call: str, status: int, text: str):
        super().__init__(f"{call}: status {status} ({text})")
        self.call, self.status = call, status


def library_path() -> str:
    return _LIB_PATH


def load_library(path: Optional[str] = None):
    """Open libloco.so (built by paper_2407_04480_amd.build); raises if it is not there."""
    global _lib
    if path is None and _lib is not None:
        return _lib
    p = path or _LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} not found: build it first (python -m paper_2407_04480_amd.build); there is no fallback path")
    lib = ctypes.CDLL(p)
    c = ctypes
    vp, sz, i, f = c.c_void_p, c.c_size_t, c.c_int, c.c_float
    lib.loco_status_string.argtypes, lib.loco_status_string.restype = [i], c.c_char_p
    lib.loco_code_bytes.argtypes, lib.loco_code_bytes.restype = [sz, i], sz
    lib.loco_num_blocks.argtypes, lib.loco_num_blocks.restype = [sz, i], sz
    lib.loco_set_pointer_checks.argtypes, lib.loco_set_pointer_checks.restype = [i], i
    lib.loco_error_state_init.argtypes, lib.loco_error_state_init.restype = [vp, sz, vp], i
    lib.loco_compensate_quantize.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp, vp]
    lib.loco_compensate_quantize.restype = i
    lib.loco_dequant_reduce.argtypes = [vp, sz, vp, sz, i, sz, i, i, vp, vp]
    lib.loco_dequant_reduce.restype = i
    lib.loco_compensate_quantize_bf16_scales.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp, vp]
    lib.loco_compensate_quantize_bf16_scales.restype = i
    lib.loco_dequant_reduce_bf16_scales.argtypes = [vp, sz, vp, sz, i, sz, i, i, vp, vp]
    lib.loco_dequant_reduce_bf16_scales.restype = i
    lib.loco_stream_copy.argtypes, lib.loco_stream_copy.restype = [vp, vp, sz, vp], i
    lib.loco_stream_read.argtypes, lib.loco_stream_read.restype = [vp, sz, vp, vp], i
    lib.loco_stream_fill.argtypes, lib.loco_stream_fill.restype = [vp, sz, vp], i
    lib.loco_stream_sum2.argtypes, lib.loco_stream_sum2.restype = [vp, vp, vp, sz, vp], i
    ip = ctypes.POINTER(ctypes.c_int)
    lib.loco_device_info.argtypes, lib.loco_device_info.restype = [ip, ip, ip, ip], i
    lib.loco_reset_due.argtypes, lib.loco_reset_due.restype = [c.c_longlong, c.c_longlong], i
    lib.loco_error_state8_init.argtypes, lib.loco_error_state8_init.restype = [vp, sz, vp], i
    lib.loco_compensate_quantize_fixed.argtypes = [vp, i, vp, sz, i, i, i, f, i, vp, vp]
    lib.loco_compensate_quantize_fixed.restype = i
    lib.loco_compensate_quantize_fixed_f32state.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp]
    lib.loco_compensate_quantize_fixed_f32state.restype = i
    lib.loco_dequant_reduce_fixed.argtypes = [vp, sz, i, sz, i, i, vp, vp]
    lib.loco_dequant_reduce_fixed.restype = i
    lib.loco_compensate_quantize_clip.argtypes = [vp, i, f, vp, sz, i, i, f, i, vp, vp, vp]
    lib.loco_compensate_quantize_clip.restype = i
    lib.loco_compensate_quantize_fixed_clip.argtypes = [vp, i, f, vp, sz, i, i, i, f, i, vp, vp]
    lib.loco_compensate_quantize_fixed_clip.restype = i
    lib.loco_dequant_reduce_sgd.argtypes = [vp, sz, vp, sz, i, sz, i, i, f, vp, vp]
    lib.loco_dequant_reduce_adam.argtypes = [vp, sz, vp, sz, i, sz, i, i, f, f, f, f, vp, vp, vp, vp]
    lib.loco_dequant_reduce_fixed_sgd.argtypes = [vp, sz, i, sz, i, i, f, vp, vp]
    lib.loco_dequant_reduce_fixed_adam.argtypes = [vp, sz, i, sz, i, i, f, f, f, f, vp, vp, vp, vp]
    lib.loco_dequant_reduce_bf16.argtypes = [vp, sz, vp, sz, i, sz, i, i, vp, vp]
    lib.loco_dequant_reduce_bf16.restype = i
    lib.loco_dequant_reduce_fixed_bf16.argtypes = [vp, sz, i, sz, i, i, vp, vp]
    lib.loco_dequant_reduce_fixed_bf16.restype = i
    i64 = c.c_int64
    lib.loco_compensate_quantize_scheduled.argtypes = [vp, i, vp, sz, i, i, f, vp, i64, vp, vp, vp]
    lib.loco_compensate_quantize_scheduled.restype = i
    lib.loco_compensate_quantize_fixed_scheduled.argtypes = [vp, i, vp, sz, i, i, i, f, vp, i64, vp, vp]
    lib.loco_compensate_quantize_fixed_scheduled.restype = i
    lib.loco_compensate_quantize_fixed_f32state_scheduled.argtypes = [vp, i, vp, sz, i, i, f, vp, i64, vp, vp]
    lib.loco_compensate_quantize_fixed_f32state_scheduled.restype = i
    lib.loco_step_index_set.argtypes, lib.loco_step_index_set.restype = [vp, i64, vp], i
    lib.loco_step_index_advance.argtypes, lib.loco_step_index_advance.restype = [vp, vp], i
    lib.loco_dequant_reduce_decomposed.argtypes = [vp, sz, vp, sz, i, sz, i, i, vp, i, vp]
    lib.loco_dequant_reduce_decomposed.restype = i
    lib.loco_dequant_reduce_decomposition.argtypes, lib.loco_dequant_reduce_decomposition.restype = [i, i, i], i
    lib.loco_runtime_copy.argtypes, lib.loco_runtime_copy.restype = [vp, vp, sz, vp], i
    lib.loco_compensate_quantize_staged_codes.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp, vp]
    lib.loco_compensate_quantize_staged_codes.restype = i
    lib.loco_compensate_quantize_resident.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp, i, vp]
    lib.loco_compensate_quantize_resident.restype = i
    lib.loco_stream_update3.argtypes, lib.loco_stream_update3.restype = [vp, vp, vp, sz, vp], i
    for _n in ("loco_dequant_reduce_sgd", "loco_dequant_reduce_adam", "loco_dequant_reduce_fixed_sgd",
               "loco_dequant_reduce_fixed_adam"):
        getattr(lib, _n).restype = i
    if path is None:
        _lib = lib
    return lib


def _check(call: str, status: int):
    if status != LOCO_OK:
        raise LocoError(call, status, load_library().loco_status_string(status).decode())


def _dev_ptr(t: torch.Tensor, name: str, dtype=None) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a torch tensor on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream_handle(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def loco_code_bytes(n: int, bits: int) -> int:
    return load_library().loco_code_bytes(n, bits)


def loco_num_blocks(n: int, block_size: int) -> int:
    return load_library().loco_num_blocks(n, block_size)


def loco_set_pointer_checks(enabled: bool) -> bool:
    return bool(load_library().loco_set_pointer_checks(1 if enabled else 0))


def loco_error_state_init(err_state: torch.Tensor, stream=None) -> None:
    """e~_0 = 0 (below Eq. 5 of arXiv 2407.04480); also the hard reset of Eq. 7."""
    lib = load_library()
    p = _dev_ptr(err_state, "err_state", torch.float32)
    _check("loco_error_state_init", lib.loco_error_state_init(p, err_state.numel(), _stream_handle(stream)))


def loco_compensate_quantize_clip(grad, clip_abs: float, err_state, bits, block_size, beta, reset, codes_out,
                                  scales_out, stream=None) -> None:
    """loco_compensate_quantize with the gradient clipped element-wise to [-clip_abs, clip_abs] first."""
    loco_compensate_quantize(grad, err_state, bits, block_size, beta, reset, codes_out, scales_out, stream,
                             _clip_abs=float(clip_abs))


def loco_compensate_quantize_fixed_clip(grad, clip_abs: float, err_state8, bits, log2_s, se_mult, beta, reset,
                                        codes_out, stream=None) -> None:
    """loco_compensate_quantize_fixed with the gradient clipped to [-clip_abs, clip_abs] first."""
    loco_compensate_quantize_fixed(grad, err_state8, bits, log2_s, se_mult, beta, reset, codes_out, stream,
                                   _clip_abs=float(clip_abs))


def loco_compensate_quantize(grad: torch.Tensor, err_state: torch.Tensor, bits: int, block_size: int,
                             beta: float, reset: bool, codes_out: torch.Tensor, scales_out: torch.Tensor,
                             stream=None, _clip_abs=None, _bf16_scales=False) -> None:
    """Algorithm 1 steps 1-2 (Eq. 1-5, 7): err_state is updated in place, codes_out
    (uint8) and scales_out (float32) receive the payload."""
    lib = load_library()
    if grad.dtype == torch.float32:
        gd = LOCO_F32
    elif grad.dtype == torch.bfloat16:
        gd = LOCO_BF16
    else:
        raise TypeError(f"grad must be float32 or bfloat16, got {grad.dtype}")
    n = grad.numel()
    pg = _dev_ptr(grad, "grad")
    pe = _dev_ptr(err_state, "err_state", torch.float32)
    pc = _dev_ptr(codes_out, "codes_out", torch.uint8)
    ps = _dev_ptr(scales_out, "scales_out", torch.bfloat16 if _bf16_scales else torch.float32)
    if err_state.numel() != n:
        raise ValueError("err_state must have as many elements as grad")
    if bits in (4, 8) and block_size >= 1:
        if codes_out.numel() < (n * bits + 7) // 8:
            raise ValueError("codes_out too small")
        if scales_out.numel() < (n + block_size - 1) // block_size:
            raise ValueError("scales_out too small")
    if _bf16_scales:
        if _clip_abs is not None:
            raise ValueError("bf16 block steps are offered without clipping")
        st = lib.loco_compensate_quantize_bf16_scales(pg, gd, pe, n, int(bits), int(block_size), float(beta),
                                                      1 if reset else 0, pc, ps, _stream_handle(stream))
        _check("loco_compensate_quantize_bf16_scales", st)
    elif _clip_abs is None:
        st = lib.loco_compensate_quantize(pg, gd, pe, n, int(bits), int(block_size), float(beta),
                                          1 if reset else 0, pc, ps, _stream_handle(stream))
        _check("loco_compensate_quantize", st)
    else:
        st = lib.loco_compensate_quantize_clip(pg, gd, _clip_abs, pe, n, int(bits), int(block_size), float(beta),
                                               1 if reset else 0, pc, ps, _stream_handle(stream))
        _check("loco_compensate_quantize_clip", st)


def loco_dequant_reduce(codes: torch.Tensor, code_stride_bytes: int, scales: torch.Tensor,
                        scale_stride_elems: int, num_workers: int, n: int, bits: int, block_size: int,
                        grad_out: torch.Tensor, stream=None, _bf16_scales=False) -> None:
    """Algorithm 1 step 3 / Eq. 8: decode num_workers payloads and average into grad_out (float32)."""
    lib = load_library()
    pc = _dev_ptr(codes, "codes", torch.uint8)
    ps = _dev_ptr(scales, "scales", torch.bfloat16 if _bf16_scales else torch.float32)
    po = _dev_ptr(grad_out, "grad_out", torch.float32)
    if grad_out.numel() < n:
        raise ValueError("grad_out too small")
    if bits in (4, 8) and block_size >= 1 and num_workers >= 1 and n > 0:
        cs = code_stride_bytes if num_workers > 1 else 0
        ss = scale_stride_elems if num_workers > 1 else 0
        if codes.numel() < (num_workers - 1) * cs + (n * bits + 7) // 8:
            raise ValueError("codes too small for num_workers payloads at this stride")
        if scales.numel() < (num_workers - 1) * ss + (n + block_size - 1) // block_size:
            raise ValueError("scales too small for num_workers payloads at this stride")
    name = "loco_dequant_reduce_bf16_scales" if _bf16_scales else "loco_dequant_reduce"
    st = getattr(lib, name)(pc, int(code_stride_bytes), ps, int(scale_stride_elems), int(num_workers),
                            int(n), int(bits), int(block_size), po, _stream_handle(stream))
    _check(name, st)


def loco_compensate_quantize_bf16_scales(grad, err_state, bits, block_size, beta, reset, codes_out,
                                         scales_out, stream=None) -> None:
    """Algorithm 1 steps 1-2 with the block steps rounded to bf16 before use; scales_out is bfloat16."""
    loco_compensate_quantize(grad, err_state, bits, block_size, beta, reset, codes_out, scales_out, stream,
                             _bf16_scales=True)


def loco_dequant_reduce_bf16_scales(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits,
                                    block_size, grad_out, stream=None) -> None:
    """Eq. 8 over payloads whose block steps are bfloat16."""
    loco_dequant_reduce(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                        grad_out, stream, _bf16_scales=True)


def loco_stream_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """Plain device copy with the kernels' load/store shape (measurement aid)."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst too small")
    st = lib.loco_stream_copy(_dev_ptr(dst, "dst"), _dev_ptr(src, "src"), nbytes, _stream_handle(stream))
    _check("loco_stream_copy", st)


def loco_stream_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Reads all of src and writes (almost) nothing: the pure-read ceiling (measurement aid)."""
    lib = load_library()
    if sink.numel() * sink.element_size() < 16:
        raise ValueError("sink must hold 16 bytes")
    st = lib.loco_stream_read(_dev_ptr(src, "src"), src.numel() * src.element_size(), _dev_ptr(sink, "sink"),
                              _stream_handle(stream))
    _check("loco_stream_read", st)


def loco_stream_fill(dst: torch.Tensor, stream=None) -> None:
    """Zero fill with the kernels' store shape: the pure-write ceiling (measurement aid)."""
    lib = load_library()
    st = lib.loco_stream_fill(_dev_ptr(dst, "dst"), dst.numel() * dst.element_size(), _stream_handle(stream))
    _check("loco_stream_fill", st)


def loco_stream_sum2(dst: torch.Tensor, src_a: torch.Tensor, src_b: torch.Tensor, stream=None) -> None:
    """dst = src_a + src_b on 32-bit words: two read streams and one write stream (measurement aid)."""
    lib = load_library()
    nbytes = src_a.numel() * src_a.element_size()
    if src_b.numel() * src_b.element_size() != nbytes or dst.numel() * dst.element_size() < nbytes:
        raise ValueError("sizes differ")
    st = lib.loco_stream_sum2(_dev_ptr(dst, "dst"), _dev_ptr(src_a, "src_a"), _dev_ptr(src_b, "src_b"), nbytes,
                              _stream_handle(stream))
    _check("loco_stream_sum2", st)


def loco_device_info() -> dict:
    """What the current device reports: memory clock, bus width, unit count (measurement aid)."""
    lib = load_library()
    vals = [ctypes.c_int(0) for _ in range(4)]
    st = lib.loco_device_info(*[ctypes.byref(v) for v in vals])
    _check("loco_device_info", st)
    keys = ("memory_clock_khz", "memory_bus_bits", "compute_units", "engine_clock_khz")
    return {k: v.value for k, v in zip(keys, vals)}


def loco_reset_due(step_index: int, reset_period: int) -> bool:
    """Eq. 7 of arXiv 2407.04480: is step k a reset step (k % T_c == 0)?"""
    return bool(load_library().loco_reset_due(int(step_index), int(reset_period)))


def loco_error_state8_init(err_state8: torch.Tensor, stream=None) -> None:
    """e_0 = 0 for the 8-bit error state of Algorithm 1 as printed."""
    lib = load_library()
    p = _dev_ptr(err_state8, "err_state8", torch.int8)
    _check("loco_error_state8_init", lib.loco_error_state8_init(p, err_state8.numel(), _stream_handle(stream)))


def loco_compensate_quantize_fixed_f32state(grad: torch.Tensor, err_state: torch.Tensor, bits: int, log2_s: int,
                                            beta: float, reset: bool, codes_out: torch.Tensor, stream=None) -> None:
    """Algorithm 1 steps 1-2 with the global scale s = 2^log2_s and the compensation error kept
    in float32 (the ablation row without error compression): err_state is updated in place."""
    lib = load_library()
    if grad.dtype == torch.float32:
        gd = LOCO_F32
    elif grad.dtype == torch.bfloat16:
        gd = LOCO_BF16
    else:
        raise TypeError(f"grad must be float32 or bfloat16, got {grad.dtype}")
    n = grad.numel()
    pg = _dev_ptr(grad, "grad")
    pe = _dev_ptr(err_state, "err_state", torch.float32)
    pc = _dev_ptr(codes_out, "codes_out", torch.uint8)
    if err_state.numel() != n:
        raise ValueError("err_state must have as many elements as grad")
    if bits in (4, 8) and codes_out.numel() < (n * bits + 7) // 8:
        raise ValueError("codes_out too small")
    st = lib.loco_compensate_quantize_fixed_f32state(pg, gd, pe, n, int(bits), int(log2_s), float(beta),
                                                     1 if reset else 0, pc, _stream_handle(stream))
    _check("loco_compensate_quantize_fixed_f32state", st)


def loco_compensate_quantize_fixed(grad: torch.Tensor, err_state8: torch.Tensor, bits: int, log2_s: int,
                                   se_mult: int, beta: float, reset: bool, codes_out: torch.Tensor,
                                   stream=None, _clip_abs=None) -> None:
    """Algorithm 1 steps 1-2 with the global scale s = 2^log2_s and the 8-bit error state
    (scale se_mult * s), Eq. 1-3, 5, 7: err_state8 (int8) is updated in place."""
    lib = load_library()
    if grad.dtype == torch.float32:
        gd = LOCO_F32
    elif grad.dtype == torch.bfloat16:
        gd = LOCO_BF16
    else:
        raise TypeError(f"grad must be float32 or bfloat16, got {grad.dtype}")
    n = grad.numel()
    pg = _dev_ptr(grad, "grad")
    pe = _dev_ptr(err_state8, "err_state8", torch.int8)
    pc = _dev_ptr(codes_out, "codes_out", torch.uint8)
    if err_state8.numel() != n:
        raise ValueError("err_state8 must have as many elements as grad")
    if bits in (4, 8) and codes_out.numel() < (n * bits + 7) // 8:
        raise ValueError("codes_out too small")
    if _clip_abs is None:
        st = lib.loco_compensate_quantize_fixed(pg, gd, pe, n, int(bits), int(log2_s), int(se_mult), float(beta),
                                                1 if reset else 0, pc, _stream_handle(stream))
        _check("loco_compensate_quantize_fixed", st)
    else:
        st = lib.loco_compensate_quantize_fixed_clip(pg, gd, _clip_abs, pe, n, int(bits), int(log2_s), int(se_mult),
                                                     float(beta), 1 if reset else 0, pc, _stream_handle(stream))
        _check("loco_compensate_quantize_fixed_clip", st)


def loco_dequant_reduce_fixed(codes: torch.Tensor, code_stride_bytes: int, num_workers: int, n: int, bits: int,
                              log2_s: int, grad_out: torch.Tensor, stream=None) -> None:
    """Algorithm 1 step 3 / Eq. 8 with the global scale."""
    lib = load_library()
    pc = _dev_ptr(codes, "codes", torch.uint8)
    po = _dev_ptr(grad_out, "grad_out", torch.float32)
    if grad_out.numel() < n:
        raise ValueError("grad_out too small")
    if bits in (4, 8) and num_workers >= 1 and n > 0:
        cs = code_stride_bytes if num_workers > 1 else 0
        if codes.numel() < (num_workers - 1) * cs + (n * bits + 7) // 8:
            raise ValueError("codes too small for num_workers payloads at this stride")
    st = lib.loco_dequant_reduce_fixed(pc, int(code_stride_bytes), int(num_workers), int(n), int(bits),
                                       int(log2_s), po, _stream_handle(stream))
    _check("loco_dequant_reduce_fixed", st)


def _f32(t, name, n):
    p = _dev_ptr(t, name, torch.float32)
    if t.numel() < n:
        raise ValueError(f"{name} too small")
    return p


def loco_dequant_reduce_sgd(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                            eta: float, theta: torch.Tensor, stream=None) -> None:
    """Eq. 8 fused with the SGD step of Eq. 9: theta <- theta - eta * g~ (in place)."""
    lib = load_library()
    st = lib.loco_dequant_reduce_sgd(_dev_ptr(codes, "codes", torch.uint8), int(code_stride_bytes),
                                     _dev_ptr(scales, "scales", torch.float32), int(scale_stride_elems),
                                     int(num_workers), int(n), int(bits), int(block_size), float(eta),
                                     _f32(theta, "theta", n), _stream_handle(stream))
    _check("loco_dequant_reduce_sgd", st)


def loco_dequant_reduce_adam(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                             eta: float, beta1: float, beta2: float, delta: float, m: torch.Tensor,
                             v: torch.Tensor, theta: torch.Tensor, stream=None) -> None:
    """Eq. 8 fused with the Adam-family step of Eq. 10 (m, v, theta updated in place)."""
    lib = load_library()
    st = lib.loco_dequant_reduce_adam(_dev_ptr(codes, "codes", torch.uint8), int(code_stride_bytes),
                                      _dev_ptr(scales, "scales", torch.float32), int(scale_stride_elems),
                                      int(num_workers), int(n), int(bits), int(block_size), float(eta),
                                      float(beta1), float(beta2), float(delta), _f32(m, "m", n), _f32(v, "v", n),
                                      _f32(theta, "theta", n), _stream_handle(stream))
    _check("loco_dequant_reduce_adam", st)


def loco_dequant_reduce_fixed_sgd(codes, code_stride_bytes, num_workers, n, bits, log2_s, eta: float,
                                  theta: torch.Tensor, stream=None) -> None:
    """Eq. 8 with the global scale fused with Eq. 9."""
    lib = load_library()
    st = lib.loco_dequant_reduce_fixed_sgd(_dev_ptr(codes, "codes", torch.uint8), int(code_stride_bytes),
                                           int(num_workers), int(n), int(bits), int(log2_s), float(eta),
                                           _f32(theta, "theta", n), _stream_handle(stream))
    _check("loco_dequant_reduce_fixed_sgd", st)


def loco_dequant_reduce_fixed_adam(codes, code_stride_bytes, num_workers, n, bits, log2_s, eta: float, beta1: float,
                                   beta2: float, delta: float, m: torch.Tensor, v: torch.Tensor,
                                   theta: torch.Tensor, stream=None) -> None:
    """Eq. 8 with the global scale fused with Eq. 10."""
    lib = load_library()
    st = lib.loco_dequant_reduce_fixed_adam(_dev_ptr(codes, "codes", torch.uint8), int(code_stride_bytes),
                                            int(num_workers), int(n), int(bits), int(log2_s), float(eta),
                                            float(beta1), float(beta2), float(delta), _f32(m, "m", n),
                                            _f32(v, "v", n), _f32(theta, "theta", n), _stream_handle(stream))
    _check("loco_dequant_reduce_fixed_adam", st)


def loco_dequant_reduce_bf16(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                             grad_out: torch.Tensor, stream=None) -> None:
    """Eq. 8 with the result rounded to bf16 (grad_out: torch.bfloat16)."""
    lib = load_library()
    po = _dev_ptr(grad_out, "grad_out", torch.bfloat16)
    if grad_out.numel() < n:
        raise ValueError("grad_out too small")
    st = lib.loco_dequant_reduce_bf16(_dev_ptr(codes, "codes", torch.uint8), int(code_stride_bytes),
                                      _dev_ptr(scales, "scales", torch.float32), int(scale_stride_elems),
                                      int(num_workers), int(n), int(bits), int(block_size), po,
                                      _stream_handle(stream))
    _check("loco_dequant_reduce_bf16", st)


def loco_dequant_reduce_fixed_bf16(codes, code_stride_bytes, num_workers, n, bits, log2_s, grad_out: torch.Tensor,
                                   stream=None) -> None:
    """Eq. 8 with the global scale, result rounded to bf16."""
    lib = load_library()
    po = _dev_ptr(grad_out, "grad_out", torch.bfloat16)
    if grad_out.numel() < n:
        raise ValueError("grad_out too small")
    st = lib.loco_dequant_reduce_fixed_bf16(_dev_ptr(codes, "codes", torch.uint8), int(code_stride_bytes),
                                            int(num_workers), int(n), int(bits), int(log2_s), po,
                                            _stream_handle(stream))
    _check("loco_dequant_reduce_fixed_bf16", st)


def _grad_dtype_code(grad: torch.Tensor) -> int:
    if grad.dtype == torch.float32:
        return LOCO_F32
    if grad.dtype == torch.bfloat16:
        return LOCO_BF16
    raise TypeError(f"grad must be float32 or bfloat16, got {grad.dtype}")


def _step_index_ptr(step_index: torch.Tensor) -> int:
    p = _dev_ptr(step_index, "step_index", torch.int64)
    if step_index.numel() != 1:
        raise ValueError("step_index must hold exactly one int64")
    return p


def loco_step_index_set(step_index: torch.Tensor, value: int, stream=None) -> None:
    """k = value for the step counter of the _scheduled calls (one int64 on the GPU)."""
    lib = load_library()
    _check("loco_step_index_set", lib.loco_step_index_set(_step_index_ptr(step_index), int(value),
                                                          _stream_handle(stream)))


def loco_step_index_advance(step_index: torch.Tensor, stream=None) -> None:
    """k = k + 1 (a small kernel, so the call can sit inside a captured HIP graph)."""
    lib = load_library()
    _check("loco_step_index_advance", lib.loco_step_index_advance(_step_index_ptr(step_index), _stream_handle(stream)))


def loco_compensate_quantize_scheduled(grad, err_state, bits, block_size, beta, step_index: torch.Tensor,
                                       reset_period: int, codes_out, scales_out, stream=None) -> None:
    """Algorithm 1 steps 1-2 with Eq. 7's reset schedule (k % reset_period == 0) evaluated in the
    kernel from the step counter in device memory."""
    lib = load_library()
    n = grad.numel()
    if err_state.numel() != n:
        raise ValueError("err_state must have as many elements as grad")
    if bits in (4, 8) and block_size >= 1:
        if codes_out.numel() < (n * bits + 7) // 8:
            raise ValueError("codes_out too small")
        if scales_out.numel() < (n + block_size - 1) // block_size:
            raise ValueError("scales_out too small")
    st = lib.loco_compensate_quantize_scheduled(
        _dev_ptr(grad, "grad"), _grad_dtype_code(grad), _dev_ptr(err_state, "err_state", torch.float32), n, int(bits),
        int(block_size), float(beta), _step_index_ptr(step_index), int(reset_period),
        _dev_ptr(codes_out, "codes_out", torch.uint8), _dev_ptr(scales_out, "scales_out", torch.float32),
        _stream_handle(stream))
    _check("loco_compensate_quantize_scheduled", st)


def loco_compensate_quantize_fixed_scheduled(grad, err_state8, bits, log2_s, se_mult, beta, step_index: torch.Tensor,
                                             reset_period: int, codes_out, stream=None) -> None:
    """Algorithm 1 as printed (global scale, 8-bit error state) with Eq. 7's schedule on the device."""
    lib = load_library()
    n = grad.numel()
    if err_state8.numel() != n:
        raise ValueError("err_state8 must have as many elements as grad")
    if bits in (4, 8) and codes_out.numel() < (n * bits + 7) // 8:
        raise ValueError("codes_out too small")
    st = lib.loco_compensate_quantize_fixed_scheduled(
        _dev_ptr(grad, "grad"), _grad_dtype_code(grad), _dev_ptr(err_state8, "err_state8", torch.int8), n, int(bits),
        int(log2_s), int(se_mult), float(beta), _step_index_ptr(step_index), int(reset_period),
        _dev_ptr(codes_out, "codes_out", torch.uint8), _stream_handle(stream))
    _check("loco_compensate_quantize_fixed_scheduled", st)


def loco_compensate_quantize_fixed_f32state_scheduled(grad, err_state, bits, log2_s, beta, step_index: torch.Tensor,
                                                      reset_period: int, codes_out, stream=None) -> None:
    """Global scale, fp32 compensation error, Eq. 7's schedule on the device."""
    lib = load_library()
    n = grad.numel()
    if err_state.numel() != n:
        raise ValueError("err_state must have as many elements as grad")
    if bits in (4, 8) and codes_out.numel() < (n * bits + 7) // 8:
        raise ValueError("codes_out too small")
    st = lib.loco_compensate_quantize_fixed_f32state_scheduled(
        _dev_ptr(grad, "grad"), _grad_dtype_code(grad), _dev_ptr(err_state, "err_state", torch.float32), n, int(bits),
        int(log2_s), float(beta), _step_index_ptr(step_index), int(reset_period),
        _dev_ptr(codes_out, "codes_out", torch.uint8), _stream_handle(stream))
    _check("loco_compensate_quantize_fixed_f32state_scheduled", st)


def loco_dequant_reduce_decomposed(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits,
                                   block_size, grad_out, decomposition: int, stream=None) -> None:
    """loco_dequant_reduce with the work decomposition (0..5, see loco.h) chosen by the caller."""
    lib = load_library()
    pc = _dev_ptr(codes, "codes", torch.uint8)
    ps = _dev_ptr(scales, "scales", torch.float32)
    po = _dev_ptr(grad_out, "grad_out", torch.float32)
    if grad_out.numel() < n:
        raise ValueError("grad_out too small")
    if bits in (4, 8) and block_size >= 1 and num_workers >= 1 and n > 0:
        cs = code_stride_bytes if num_workers > 1 else 0
        ss = scale_stride_elems if num_workers > 1 else 0
        if codes.numel() < (num_workers - 1) * cs + (n * bits + 7) // 8:
            raise ValueError("codes too small for num_workers payloads at this stride")
        if scales.numel() < (num_workers - 1) * ss + (n + block_size - 1) // block_size:
            raise ValueError("scales too small for num_workers payloads at this stride")
    st = lib.loco_dequant_reduce_decomposed(pc, int(code_stride_bytes), ps, int(scale_stride_elems), int(num_workers),
                                            int(n), int(bits), int(block_size), po, int(decomposition),
                                            _stream_handle(stream))
    _check("loco_dequant_reduce_decomposed", st)


def loco_dequant_reduce_decomposition(num_workers: int, bits: int, block_size: int) -> int:
    """The decomposition (1..5) loco_dequant_reduce picks for these arguments; -1 if unsupported."""
    return load_library().loco_dequant_reduce_decomposition(int(num_workers), int(bits), int(block_size))


def loco_runtime_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """The HIP runtime's own device-to-device copy on the stream (measurement aid)."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst too small")
    st = lib.loco_runtime_copy(_dev_ptr(dst, "dst"), _dev_ptr(src, "src"), nbytes, _stream_handle(stream))
    _check("loco_runtime_copy", st)


def loco_stream_update3(a: torch.Tensor, b: torch.Tensor, c: torch.Tensor, stream=None) -> None:
    """In-place update of three equally sized arrays: the traffic of an optimizer step alone (measurement aid)."""
    lib = load_library()
    nbytes = a.numel() * a.element_size()
    if b.numel() * b.element_size() != nbytes or c.numel() * c.element_size() != nbytes:
        raise ValueError("sizes differ")
    st = lib.loco_stream_update3(_dev_ptr(a, "a"), _dev_ptr(b, "b"), _dev_ptr(c, "c"), nbytes, _stream_handle(stream))
    _check("loco_stream_update3", st)


def loco_compensate_quantize_staged_codes(grad, err_state, bits, block_size, beta, reset, codes_out, scales_out,
                                          stream=None) -> None:
    """loco_compensate_quantize (4-bit) with the codes staged through LDS into 16-byte stores (measurement aid)."""
    lib = load_library()
    n = grad.numel()
    if err_state.numel() != n:
        raise ValueError("err_state must have as many elements as grad")
    if codes_out.numel() < (n * 4 + 7) // 8 or (block_size >= 1 and scales_out.numel() < (n + block_size - 1) // block_size):
        raise ValueError("codes_out or scales_out too small")
    st = lib.loco_compensate_quantize_staged_codes(
        _dev_ptr(grad, "grad"), _grad_dtype_code(grad), _dev_ptr(err_state, "err_state", torch.float32), n, int(bits),
        int(block_size), float(beta), 1 if reset else 0, _dev_ptr(codes_out, "codes_out", torch.uint8),
        _dev_ptr(scales_out, "scales_out", torch.float32), _stream_handle(stream))
    _check("loco_compensate_quantize_staged_codes", st)


def loco_compensate_quantize_resident(grad, err_state, bits, block_size, beta, reset, codes_out, scales_out,
                                      waves_per_simd, stream=None) -> None:
    """loco_compensate_quantize with 4, 6 or 8 wavefronts resident per SIMD (measurement aid)."""
    lib = load_library()
    n = grad.numel()
    if err_state.numel() != n:
        raise ValueError("err_state must have as many elements as grad")
    if bits in (4, 8) and block_size >= 1 and (codes_out.numel() < (n * bits + 7) // 8
                                               or scales_out.numel() < (n + block_size - 1) // block_size):
        raise ValueError("codes_out or scales_out too small")
    st = lib.loco_compensate_quantize_resident(
        _dev_ptr(grad, "grad"), _grad_dtype_code(grad), _dev_ptr(err_state, "err_state", torch.float32), n, int(bits),
        int(block_size), float(beta), 1 if reset else 0, _dev_ptr(codes_out, "codes_out", torch.uint8),
        _dev_ptr(scales_out, "scales_out", torch.float32), int(waves_per_simd), _stream_handle(stream))
    _check("loco_compensate_quantize_resident", st)
