"""Loader for the CPU oracle (oracle/loco_ref.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It builds the plain C oracle with gcc and wraps its entry points for
numpy arrays.  It imports nothing from the GPU package and the GPU package
imports nothing from here.

The functions mirror the three calls of the method (LoCo, arXiv 2407.04480,
Alg. 1): error_state_init (e~_0 = 0), compensate_quantize (steps 1-2, Eq. 1-5, 7)
and dequant_reduce (step 3, Eq. 8).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "loco_ref.c"), os.path.join(_HERE, "loco_ref_mt.c")]
_SO = os.path.join(_HERE, "libloco_ref.so")
# One rounding per written operation: no contraction, no fast-math, plain x86-64.
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall", "-Wextra"]

F32 = 0
BF16 = 1

_lock = threading.Lock()
_lib = None


def build(force: bool = False, out: str | None = None, srcs=None, extra_flags=()) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    out = out or _SO
    srcs = list(srcs or _SRCS)
    if not force and os.path.exists(out) and all(
        os.path.getmtime(out) >= os.path.getmtime(s) for s in srcs
    ):
        return out
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = ["gcc", *CFLAGS, *extra_flags, "-o", tmp, *srcs, "-lm", "-lpthread"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    os.replace(tmp, out)
    return out


def _bind(lib):
    c = ctypes
    vp, sz, i, f = c.c_void_p, c.c_size_t, c.c_int, c.c_float
    lib.loco_ref_error_state_init.argtypes = [vp, sz]
    lib.loco_ref_reset_due.argtypes = [c.c_longlong, c.c_longlong]
    lib.loco_ref_reset_due.restype = c.c_int
    lib.loco_ref_compensate_quantize.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp]
    lib.loco_ref_compensate_quantize_blocks.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp, sz, sz]
    lib.loco_ref_compensate_quantize_mt.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp, i]
    lib.loco_ref_dequant_reduce.argtypes = [vp, sz, vp, sz, i, sz, i, i, vp]
    lib.loco_ref_dequant_reduce_mt.argtypes = [vp, sz, vp, sz, i, sz, i, i, vp, i]
    lib.loco_ref_fixed_compensate_quantize.argtypes = [vp, i, vp, sz, i, i, i, f, i, vp]
    lib.loco_ref_fixed_compensate_quantize_mt.argtypes = [vp, i, vp, sz, i, i, i, f, i, vp, i]
    lib.loco_ref_fixed_compensate_quantize_f32state.argtypes = [vp, i, vp, sz, i, i, f, i, vp]
    lib.loco_ref_fixed_dequant_reduce.argtypes = [vp, sz, i, sz, i, i, vp]
    lib.loco_ref_fixed_dequant_reduce_mt.argtypes = [vp, sz, i, sz, i, i, vp, i]
    lib.loco_ref_compensate_quantize_bf16_scales.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp]
    lib.loco_ref_compensate_quantize_bf16_scales_mt.argtypes = [vp, i, vp, sz, i, i, f, i, vp, vp, i]
    lib.loco_ref_dequant_reduce_bf16_scales.argtypes = [vp, sz, vp, sz, i, sz, i, i, vp]
    lib.loco_ref_dequant_reduce_bf16_scales_mt.argtypes = [vp, sz, vp, sz, i, sz, i, i, vp, i]
    lib.loco_ref_clip_gradient.argtypes = [vp, i, sz, f, vp]
    lib.loco_ref_round_to_bf16.argtypes = [vp, sz, vp]
    lib.loco_ref_round_to_bf16.restype = c.c_int
    lib.loco_ref_sgd_update.argtypes = [vp, vp, sz, f]
    lib.loco_ref_adam_update.argtypes = [vp, vp, vp, vp, sz, f, f, f, f]
    for name in (
        "loco_ref_sgd_update",
        "loco_ref_adam_update",
        "loco_ref_clip_gradient",
        "loco_ref_fixed_compensate_quantize",
        "loco_ref_fixed_compensate_quantize_mt",
        "loco_ref_fixed_compensate_quantize_f32state",
        "loco_ref_fixed_dequant_reduce",
        "loco_ref_fixed_dequant_reduce_mt",
        "loco_ref_error_state_init",
        "loco_ref_compensate_quantize",
        "loco_ref_compensate_quantize_blocks",
        "loco_ref_compensate_quantize_mt",
        "loco_ref_dequant_reduce",
        "loco_ref_dequant_reduce_mt",
        "loco_ref_compensate_quantize_bf16_scales",
        "loco_ref_compensate_quantize_bf16_scales_mt",
        "loco_ref_dequant_reduce_bf16_scales",
        "loco_ref_dequant_reduce_bf16_scales_mt",
    ):
        getattr(lib, name).restype = c.c_int
    return lib


def load(path: str | None = None):
    """ctypes handle of the oracle library (built on first use)."""
    global _lib
    if path is not None:
        return _bind(ctypes.CDLL(path))
    with _lock:
        if _lib is None:
            _lib = _bind(ctypes.CDLL(build()))
        return _lib


def code_bytes(n: int, bits: int) -> int:
    return (n * bits + 7) // 8


def num_blocks(n: int, block_size: int) -> int:
    return (n + block_size - 1) // block_size


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _grad_dtype(grad: np.ndarray) -> int:
    if grad.dtype == np.float32:
        return F32
    if grad.dtype == np.uint16:  # bf16 bit patterns
        return BF16
    raise TypeError("grad must be float32, or uint16 holding bf16 bit patterns")


def error_state_init(err_state: np.ndarray, lib=None) -> None:
    lib = lib or load()
    assert err_state.dtype == np.float32 and err_state.flags.c_contiguous
    rc = lib.loco_ref_error_state_init(_ptr(err_state), err_state.size)
    if rc:
        raise ValueError("loco_ref_error_state_init: status %d" % rc)


def reset_due(step_index: int, reset_period: int, lib=None) -> bool:
    """Eq. 7 / Alg. 1: step k resets the state when k % T_c == 0 (never for T_c <= 0)."""
    lib = lib or load()
    return bool(lib.loco_ref_reset_due(int(step_index), int(reset_period)))


def compensate_quantize(grad, err_state, bits, block_size, beta, reset=0, threads=1, lib=None,
                        bf16_scales=False):
    """Alg. 1 steps 1-2.  err_state (float32) is updated in place.

    Returns (codes uint8[ceil(n*bits/8)], scales float32[ceil(n/block_size)]); with
    bf16_scales the steps are rounded to bf16 before use and returned as uint16 bit patterns.
    """
    lib = lib or load()
    grad = np.ascontiguousarray(grad)
    assert err_state.dtype == np.float32 and err_state.flags.c_contiguous
    n = grad.size
    assert err_state.size == n
    codes = np.zeros(code_bytes(n, bits), dtype=np.uint8)
    scales = np.zeros(num_blocks(n, block_size) if block_size >= 1 else 0,
                      dtype=np.uint16 if bf16_scales else np.float32)
    args = [_ptr(grad), _grad_dtype(grad), _ptr(err_state), n, bits, block_size,
            float(beta), int(reset), _ptr(codes), _ptr(scales)]
    suffix = "_bf16_scales" if bf16_scales else ""
    if threads > 1:
        rc = getattr(lib, "loco_ref_compensate_quantize%s_mt" % suffix)(*args, int(threads))
    else:
        rc = getattr(lib, "loco_ref_compensate_quantize" + suffix)(*args)
    if rc:
        raise ValueError("loco_ref_compensate_quantize: status %d" % rc)
    return codes, scales


def dequant_reduce(codes, scales, num_workers, n, bits, block_size,
                   code_stride_bytes=None, scale_stride_elems=None, threads=1, lib=None):
    """Alg. 1 step 3 / Eq. 8.  codes/scales hold num_workers payloads at the given strides.

    scales is float32, or uint16 holding bf16 steps.  Returns the averaged gradient, float32[n].
    """
    lib = lib or load()
    codes = np.ascontiguousarray(codes).reshape(-1)
    scales = np.ascontiguousarray(scales).reshape(-1)
    assert codes.dtype == np.uint8 and scales.dtype in (np.float32, np.uint16)
    suffix = "_bf16_scales" if scales.dtype == np.uint16 else ""
    if code_stride_bytes is None:
        code_stride_bytes = code_bytes(n, bits)
    if scale_stride_elems is None:
        scale_stride_elems = num_blocks(n, block_size)
    if num_workers >= 1 and n > 0:
        assert codes.size >= (num_workers - 1) * code_stride_bytes + code_bytes(n, bits)
        assert scales.size >= (num_workers - 1) * scale_stride_elems + num_blocks(n, block_size)
    out = np.zeros(n, dtype=np.float32)
    args = [_ptr(codes), code_stride_bytes, _ptr(scales), scale_stride_elems,
            int(num_workers), n, bits, block_size, _ptr(out)]
    if threads > 1:
        rc = getattr(lib, "loco_ref_dequant_reduce%s_mt" % suffix)(*args, int(threads))
    else:
        rc = getattr(lib, "loco_ref_dequant_reduce" + suffix)(*args)
    if rc:
        raise ValueError("loco_ref_dequant_reduce: status %d" % rc)
    return out


def fixed_compensate_quantize(grad, err_state8, bits, log2_s, se_mult, beta, reset=0, threads=1, lib=None):
    """Alg. 1 steps 1-2 as printed: global scale s = 2^log2_s, 8-bit error state with scale
    s_e = se_mult * s (Eq. 1-3, 5, 7).  err_state8 (int8) is updated in place; returns codes."""
    lib = lib or load()
    grad = np.ascontiguousarray(grad)
    assert err_state8.dtype == np.int8 and err_state8.flags.c_contiguous and err_state8.size == grad.size
    n = grad.size
    codes = np.zeros(code_bytes(n, bits), dtype=np.uint8)
    args = [_ptr(grad), _grad_dtype(grad), _ptr(err_state8), n, bits, int(log2_s), int(se_mult),
            float(beta), int(reset), _ptr(codes)]
    if threads > 1:
        rc = lib.loco_ref_fixed_compensate_quantize_mt(*args, int(threads))
    else:
        rc = lib.loco_ref_fixed_compensate_quantize(*args)
    if rc:
        raise ValueError("loco_ref_fixed_compensate_quantize: status %d" % rc)
    return codes


def fixed_compensate_quantize_f32state(grad, err_state, bits, log2_s, beta, reset=0, lib=None):
    """Alg. 1 steps 1-2 with the global scale s = 2^log2_s and the compensation error kept in
    float32 (the paper's ablation row without error compression).  err_state is updated in place;
    returns the codes."""
    lib = lib or load()
    grad = np.ascontiguousarray(grad)
    assert err_state.dtype == np.float32 and err_state.flags.c_contiguous and err_state.size == grad.size
    n = grad.size
    codes = np.zeros(code_bytes(n, bits), dtype=np.uint8)
    rc = lib.loco_ref_fixed_compensate_quantize_f32state(_ptr(grad), _grad_dtype(grad), _ptr(err_state), n,
                                                         int(bits), int(log2_s), float(beta), int(reset), _ptr(codes))
    if rc:
        raise ValueError("loco_ref_fixed_compensate_quantize_f32state: status %d" % rc)
    return codes


def fixed_dequant_reduce(codes, num_workers, n, bits, log2_s, code_stride_bytes=None, threads=1, lib=None):
    """Eq. 8 with the global scale; returns float32[n]."""
    lib = lib or load()
    codes = np.ascontiguousarray(codes).reshape(-1)
    assert codes.dtype == np.uint8
    if code_stride_bytes is None:
        code_stride_bytes = code_bytes(n, bits)
    if num_workers >= 1 and n > 0:
        assert codes.size >= (num_workers - 1) * code_stride_bytes + code_bytes(n, bits)
    out = np.zeros(n, dtype=np.float32)
    args = [_ptr(codes), code_stride_bytes, int(num_workers), n, bits, int(log2_s), _ptr(out)]
    if threads > 1:
        rc = lib.loco_ref_fixed_dequant_reduce_mt(*args, int(threads))
    else:
        rc = lib.loco_ref_fixed_dequant_reduce(*args)
    if rc:
        raise ValueError("loco_ref_fixed_dequant_reduce: status %d" % rc)
    return out


def clip_gradient(grad, clip_abs, lib=None):
    """Element-wise clipping of the local gradient to [-clip_abs, clip_abs] (Sec. 5.2); float32 out."""
    lib = lib or load()
    grad = np.ascontiguousarray(grad)
    out = np.empty(grad.size, dtype=np.float32)
    rc = lib.loco_ref_clip_gradient(_ptr(grad), _grad_dtype(grad), grad.size, float(clip_abs), _ptr(out))
    if rc:
        raise ValueError("loco_ref_clip_gradient: status %d" % rc)
    return out


def sgd_update(theta, g_avg, eta, lib=None):
    """Eq. 9: theta <- theta - eta * g~ (in place, float32)."""
    lib = lib or load()
    assert theta.dtype == np.float32 and g_avg.dtype == np.float32 and theta.size == g_avg.size
    rc = lib.loco_ref_sgd_update(_ptr(theta), _ptr(np.ascontiguousarray(g_avg)), theta.size, float(eta))
    if rc:
        raise ValueError("loco_ref_sgd_update: status %d" % rc)


def adam_update(theta, m, v, g_avg, eta, beta1, beta2, delta, lib=None):
    """Eq. 10 with Adam's pre-conditioner 1/sqrt(v + delta); theta, m, v updated in place."""
    lib = lib or load()
    for a in (theta, m, v, g_avg):
        assert a.dtype == np.float32 and a.flags.c_contiguous and a.size == theta.size
    rc = lib.loco_ref_adam_update(_ptr(theta), _ptr(m), _ptr(v), _ptr(g_avg), theta.size, float(eta),
                                  float(beta1), float(beta2), float(delta))
    if rc:
        raise ValueError("loco_ref_adam_update: status %d" % rc)


def round_to_bf16(x, lib=None):
    """float32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    lib = lib or load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.size, dtype=np.uint16)
    rc = lib.loco_ref_round_to_bf16(_ptr(x), x.size, _ptr(out))
    if rc:
        raise ValueError("loco_ref_round_to_bf16: status %d" % rc)
    return out
