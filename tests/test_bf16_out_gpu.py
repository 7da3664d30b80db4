"""Reduce with the averaged gradient written as bf16: must equal the oracle's fp32 reduce
followed by the oracle's round-to-nearest-even conversion, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import loco_dequant_reduce_bf16, loco_dequant_reduce_fixed_bf16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits_of(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


# 4-bit codes take the wide code loads (16 bytes per lane) in front of the rounding at every worker count,
# 8-bit codes the quad layout up to W = 95
@pytest.mark.parametrize("bits,B,W", [(4, 256, 8), (8, 64, 3), (4, 32, 1), (4, 512, 16), (4, 64, 20), (4, 128, 70),
                                      (4, 256, 100), (8, 64, 97)])
@pytest.mark.parametrize("n", [6 * 2048 + 777, 9, 2049])
def test_block_reduce_bf16(bits, B, W, n):
    rs = np.random.default_rng(bits + B + W + n)
    cb, nb = oracle.code_bytes(n, bits), oracle.num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    codes = rs.integers(0, 256, W * cstride, dtype=np.uint8)
    # steps chosen so that many averages fall exactly between two bf16 values
    scales = rs.choice(np.array([2.0 ** -9, 2.0 ** -10, 3e-4, 1.0, 0.0], np.float32), W * nb)
    if W <= 20:         # a few steps of 2^120 (sums stay finite): the tiles that meet one are summed again in full
        scales[rs.random(W * nb) < 0.02] = np.float32(2.0 ** 120)
    out = torch.full((n,), 7.0, dtype=torch.bfloat16, device=DEV)
    loco_dequant_reduce_bf16(torch.from_numpy(codes).to(DEV), cstride, torch.from_numpy(scales).to(DEV), nb,
                             W, n, bits, B, out)
    torch.cuda.synchronize()
    ref32 = oracle.dequant_reduce(codes, scales, W, n, bits, B, cstride, nb)
    want = oracle.round_to_bf16(ref32)
    assert np.array_equal(bits_of(out), want)
    inexact = ((ref32.view(np.uint32) & 0xFFFF) != 0).sum()
    assert W < 8 or n < 100 or inexact > 0        # the rounding is really exercised


@pytest.mark.parametrize("bits,W", [(4, 8), (8, 5), (4, 17)])
def test_fixed_reduce_bf16(bits, W):
    n, log2_s = 5 * 1024 + 301, 19
    rs = np.random.default_rng(bits * W)
    cb = oracle.code_bytes(n, bits)
    stride = (cb + 15) // 16 * 16
    codes = rs.integers(0, 256, W * stride, dtype=np.uint8)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    loco_dequant_reduce_fixed_bf16(torch.from_numpy(codes).to(DEV), stride, W, n, bits, log2_s, out)
    torch.cuda.synchronize()
    want = oracle.round_to_bf16(oracle.fixed_dequant_reduce(codes, W, n, bits, log2_s, code_stride_bytes=stride))
    assert np.array_equal(bits_of(out), want)
