"""The C-ABI library loads and exports every function include/loco.h declares (no GPU,
no compute call), and the host-only helpers agree with their definitions."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "loco.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(loco_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2407_04480_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2407_04480_amd import build
        build.build()
    return binding.load_library()


def test_header_declares_the_three_calls():
    names = declared_functions()
    for need in ("loco_error_state_init", "loco_compensate_quantize", "loco_dequant_reduce"):
        assert need in names


def test_every_declared_symbol_is_exported(lib):
    from paper_2407_04480_amd import binding
    raw = ctypes.CDLL(binding.library_path())
    for name in declared_functions():
        assert hasattr(raw, name), f"{name} declared in loco.h but not exported"
    assert sorted(binding.EXPORTS) == declared_functions()


def test_host_helpers(lib):
    from paper_2407_04480_amd import loco_code_bytes, loco_num_blocks
    for n in (0, 1, 2, 3, 255, 256, 257, 842301952, 2200000000, (1 << 40) + 1):
        assert loco_code_bytes(n, 8) == n
        assert loco_code_bytes(n, 4) == (n + 1) // 2
        for b in (32, 64, 128, 256, 512):
            assert loco_num_blocks(n, b) == (n + b - 1) // b
    assert loco_code_bytes(10, 5) == 0
    assert loco_num_blocks(10, 0) == 0
    assert lib.loco_status_string(0) == b"ok"
    assert all(lib.loco_status_string(s) for s in range(0, 7))


def test_argument_errors_need_no_gpu(lib):
    """Checks that come before any device work return their status on a box with no GPU."""
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(16)
    # bits / block size / dtype / beta
    assert lib.loco_compensate_quantize(one, 0, one, 8, 3, 256, 0.25, 0, one, one, null) == 2
    assert lib.loco_compensate_quantize(one, 0, one, 8, 4, 100, 0.25, 0, one, one, null) == 2
    assert lib.loco_compensate_quantize(one, 7, one, 8, 4, 256, 0.25, 0, one, one, null) == 2
    assert lib.loco_compensate_quantize(one, 0, one, 8, 4, 256, 1.5, 0, one, one, null) == 1
    assert lib.loco_compensate_quantize(one, 0, one, 8, 4, 256, float("nan"), 0, one, one, null) == 1
    # n == 0 is a no-op
    assert lib.loco_compensate_quantize(null, 0, null, 0, 4, 256, 0.25, 0, null, null, null) == 0
    assert lib.loco_dequant_reduce(null, 0, null, 0, 1, 0, 4, 256, null, null) == 0
    assert lib.loco_error_state_init(null, 0, null) == 0
    # NULL pointers, bad alignment, W < 1, short strides
    assert lib.loco_compensate_quantize(null, 0, one, 8, 4, 256, 0.25, 0, one, one, null) == 1
    assert lib.loco_compensate_quantize(ctypes.c_void_p(8), 0, one, 8, 4, 256, 0.25, 0, one, one, null) == 3
    assert lib.loco_dequant_reduce(one, 16, one, 1, 0, 8, 4, 256, one, null) == 1
    assert lib.loco_dequant_reduce(one, 0, one, 0, 2, 64, 4, 32, one, null) == 1
    assert lib.loco_dequant_reduce(one, 40, one, 2, 2, 64, 4, 32, one, null) == 3
    assert lib.loco_error_state_init(ctypes.c_void_p(4), 8, null) == 3
    assert lib.loco_stream_copy(one, one, 24, null) == 3
    assert lib.loco_stream_read(one, 24, one, null) == 3
    assert lib.loco_stream_fill(ctypes.c_void_p(8), 32, null) == 3
    assert lib.loco_stream_read(null, 32, one, null) == 1
    assert lib.loco_stream_fill(null, 0, null) == 0
    assert lib.loco_stream_sum2(one, one, null, 32, null) == 1
    # the integer sums of the fixed-scale reduce are exact only below 2^24: worker count bounded
    assert lib.loco_dequant_reduce_fixed(one, 16, (1 << 21) + 1, 0, 4, 19, one, null) == 2
    assert lib.loco_dequant_reduce_fixed(one, 16, (1 << 17) + 1, 0, 8, 19, one, null) == 2
    assert lib.loco_dequant_reduce_fixed(null, 16, 1 << 21, 0, 4, 19, null, null) == 0
    assert lib.loco_dequant_reduce_fixed(null, 16, 1 << 17, 0, 8, 19, null, null) == 0
    # scheduled calls: NULL or misaligned step index, negative period; decomposition out of range
    assert lib.loco_compensate_quantize_scheduled(one, 0, one, 8, 4, 256, 0.25, null, 3, one, one, null) == 1
    assert lib.loco_compensate_quantize_scheduled(one, 0, one, 8, 4, 256, 0.25, ctypes.c_void_p(12), 3, one, one, null) == 3
    assert lib.loco_compensate_quantize_scheduled(one, 0, one, 8, 4, 256, 0.25, one, -2, one, one, null) == 1
    assert lib.loco_compensate_quantize_scheduled(null, 0, null, 0, 4, 256, 0.25, null, 3, null, null, null) == 0
    assert lib.loco_step_index_advance(null, null) == 1 and lib.loco_step_index_set(ctypes.c_void_p(4), 0, null) == 3
    assert lib.loco_dequant_reduce_decomposed(one, 16, one, 1, 1, 8, 4, 256, one, 6, null) == 2
    assert lib.loco_dequant_reduce_decomposed(one, 16, one, 1, 1, 8, 4, 256, one, -1, null) == 2
    assert lib.loco_dequant_reduce_decomposition(8, 4, 256) == 1 and lib.loco_dequant_reduce_decomposition(128, 8, 64) == 5 and lib.loco_dequant_reduce_decomposition(8, 5, 256) == -1
    assert lib.loco_reset_due(0, 512) == 1 and lib.loco_reset_due(512, 512) == 1 and lib.loco_reset_due(5, 512) == 0
    assert lib.loco_runtime_copy(null, one, 16, null) == 1 and lib.loco_runtime_copy(null, null, 0, null) == 0
    # the residency variant exists for 4, 6 and 8 wavefronts per SIMD only
    assert lib.loco_compensate_quantize_resident(one, 0, one, 8, 4, 256, 0.25, 0, one, one, 5, null) == 2
    assert lib.loco_compensate_quantize_resident(null, 0, null, 0, 4, 256, 0.25, 0, null, null, 8, null) == 0
    # sizes no device can hold, and strides whose W payloads would wrap the address space
    assert lib.loco_compensate_quantize(one, 0, one, (1 << 48) + 1, 4, 256, 0.25, 0, one, one, null) == 2
    assert lib.loco_dequant_reduce(one, 1 << 50, one, 1 << 50, 2, (1 << 48) + 1, 4, 256, one, null) == 2
    assert lib.loco_dequant_reduce(one, 1 << 62, one, 1, 5, 8, 4, 256, one, null) == 1
    assert lib.loco_dequant_reduce(one, 16, one, 1 << 61, 9, 8, 4, 256, one, null) == 1
    assert lib.loco_dequant_reduce_fixed(one, 1 << 62, 5, 8, 4, 19, one, null) == 1


def test_missing_library_is_an_error(tmp_path):
    from paper_2407_04480_amd import binding
    with pytest.raises(FileNotFoundError):
        binding.load_library(str(tmp_path / "nope.so"))


def test_cpu_tensor_is_rejected(lib):
    import torch
    from paper_2407_04480_amd import loco_error_state_init
    with pytest.raises(TypeError):
        loco_error_state_init(torch.zeros(8))
