"""Element-wise gradient clipping fused in front of compensate-quantize (both forms):
the GPU call must equal the oracle's clip followed by the oracle's compensate-quantize."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize, loco_compensate_quantize_clip,
                                  loco_compensate_quantize_fixed_clip, loco_num_blocks, workloads)
from paper_2407_04480_amd.binding import LocoError

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("bits,B", [(4, 256), (8, 64), (4, 32), (4, 512)])
def test_block_form_with_clip(dtype, bits, B):
    n = 7 * 2048 + 333
    rng = torch.Generator().manual_seed(bits * B)
    e_t = torch.zeros(n, dtype=torch.float32, device=DEV)
    e_h = np.zeros(n, np.float32)
    for step, c in enumerate((1e-3, 7.7e-4, 2.0 ** -11, float("inf"))):
        g = (torch.randn(n, generator=rng) * 1e-3).to(dtype)
        codes = torch.empty(loco_code_bytes(n, bits), dtype=torch.uint8, device=DEV)
        scales = torch.empty(loco_num_blocks(n, B), dtype=torch.float32, device=DEV)
        loco_compensate_quantize_clip(g.to(DEV), c, e_t, bits, B, 0.25, False, codes, scales)
        gc = oracle.clip_gradient(workloads.as_numpy_grad(g), c)
        c_ref, s_ref = oracle.compensate_quantize(gc, e_h, bits, B, 0.25)
        torch.cuda.synchronize()
        assert np.array_equal(codes.cpu().numpy(), c_ref), f"step {step}"
        assert np.array_equal(scales.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
        assert np.array_equal(e_t.cpu().numpy(), e_h)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("bits,mult", [(4, 4), (4, 6), (8, 6)])
def test_fixed_form_with_clip(dtype, bits, mult):
    n, log2_s = 5 * 1024 + 77, 19
    s = 2.0 ** log2_s
    rng = torch.Generator().manual_seed(bits + mult)
    e_t = torch.zeros(n, dtype=torch.int8, device=DEV)
    e_h = np.zeros(n, np.int8)
    for step, c in enumerate((6.0 / s, 2.5 / s, 100.0 / s, float("inf"))):
        g = (torch.randn(n, generator=rng) * (5.0 / s)).to(dtype)
        codes = torch.empty(loco_code_bytes(n, bits), dtype=torch.uint8, device=DEV)
        loco_compensate_quantize_fixed_clip(g.to(DEV), c, e_t, bits, log2_s, mult, 0.25, False, codes)
        gc = oracle.clip_gradient(workloads.as_numpy_grad(g), c)
        c_ref = oracle.fixed_compensate_quantize(gc, e_h, bits, log2_s, mult, 0.25)
        torch.cuda.synchronize()
        assert np.array_equal(codes.cpu().numpy(), c_ref), f"step {step}"
        assert np.array_equal(e_t.cpu().numpy(), e_h)


def test_clip_rejects_bad_threshold_and_inf_equals_plain():
    n = 4096
    g = torch.randn(n, device=DEV) * 1e-3
    codes = torch.empty(n // 2, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n // 256, device=DEV)
    for bad in (0.0, -1.0, float("nan")):
        with pytest.raises(LocoError) as ei:
            loco_compensate_quantize_clip(g, bad, torch.zeros(n, device=DEV), 4, 256, 0.25, False, codes, scales)
        assert ei.value.status == 1
    e1, e2 = torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    c2, s2 = torch.empty_like(codes), torch.empty_like(scales)
    loco_compensate_quantize_clip(g, float("inf"), e1, 4, 256, 0.25, False, codes, scales)
    loco_compensate_quantize(g, e2, 4, 256, 0.25, False, c2, s2)
    torch.cuda.synchronize()
    assert torch.equal(codes, c2) and torch.equal(scales, s2) and torch.equal(e1, e2)
