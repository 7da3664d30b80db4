"""The build's device pass: the packed-fp32 feature is really off (no v_pk_*_f32 instruction in
any kernel), no kernel spills to scratch memory, and nothing writes through the scalar data
cache.  The assembly is that of this repository's own kernels, made by hipcc -S here on the CPU."""
import re

import pytest

from paper_2407_04480_amd import build


@pytest.fixture(scope="module")
def asm():
    return build.device_assembly()


def test_no_packed_fp32_instructions(asm):
    found = sorted(set(re.findall(r"\bv_pk_(?:add|mul|fma)_f32\b", asm)))
    assert not found, f"packed fp32 instructions selected: {found}"
    assert "v_fma_f32" in asm or "v_fmac_f32" in asm      # the assembly is really there (Eq. 5's fmaf)


def test_the_flag_is_what_keeps_them_out(tmp_path):
    """Without the feature flag the same compiler does select packed fp32 for plain float2 code."""
    src = tmp_path / "probe.hip"
    src.write_text("#include <hip/hip_runtime.h>\n__global__ void k(float2* a, const float2* b, float s) {\n"
                   "  int i = threadIdx.x; float2 x = a[i], y = b[i]; x.x = x.x * s + y.x; x.y = x.y * s + y.y; a[i] = x; }\n")
    with_flag = build.device_assembly(str(src))
    assert not re.search(r"\bv_pk_(?:add|mul|fma)_f32\b", with_flag)
    import subprocess
    plain = subprocess.run([build.hipcc_path(), "--offload-arch=gfx950", "-O3", "-S", "--cuda-device-only", "-o", "-", str(src)],
                           capture_output=True, text=True).stdout
    assert re.search(r"\bv_pk_(?:add|mul|fma)_f32\b", plain), "the probe no longer shows what the flag prevents"


def test_no_kernel_uses_scratch_memory(asm):
    sizes = [int(x) for x in re.findall(r"\.private_segment_fixed_size:\s*(\d+)", asm)]
    assert sizes and max(sizes) == 0, f"a kernel spills: private segment sizes {sorted(set(sizes))}"


def test_no_writes_through_the_scalar_cache(asm):
    body = "\n".join(line for line in asm.splitlines() if not line.lstrip().startswith((";", "//")))
    assert not re.search(r"\bs_(?:buffer_|scratch_)?store_|\bs_atomic_|\bs_buffer_atomic_|\bs_dcache_(?:wb|inv|discard)", body)


def test_host_note_filter():
    note = build.HOST_FEATURE_NOTE
    assert build.without_host_feature_note(f"{note}\nwarning: x\n{note}\n") == "warning: x\n"
