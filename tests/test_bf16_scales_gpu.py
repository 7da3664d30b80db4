"""Block steps kept in bf16: the GPU payload (codes, bf16 steps), the error state and the
reduce must equal the oracle's bf16-step form bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (LocoError, loco_compensate_quantize_bf16_scales,
                                  loco_dequant_reduce_bf16_scales)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FLT_MIN = np.float32(np.finfo(np.float32).tiny)


def u16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def make_grad(rs, n, B, dtype):
    g = (rs.standard_t(3, n) * 10.0 ** rs.uniform(-5, -2)).astype(np.float32)
    if n >= 4 * B:
        g[B:2 * B] = 0.0                                         # a zero block
        g[2 * B:3 * B] = 0.0
        g[2 * B] = np.float32(7) * FLT_MIN * np.float32(0.25)     # subnormal step, stays dead
        g[3 * B:4 * B] *= np.float32(1e-30)                       # tiny but live
    if dtype == "bf16":
        t = torch.from_numpy(g).to(torch.bfloat16)
        return t, u16(t)
    return torch.from_numpy(g), g


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("bits,B", [(4, 256), (8, 64), (4, 32), (8, 512), (4, 128), (8, 256)])
@pytest.mark.parametrize("n", [7 * 2048 + 301, 2048, 37])
def test_compensate_quantize_bf16_scales(dtype, bits, B, n):
    rs = np.random.default_rng(bits * 1000 + B + n)
    cb, nb = oracle.code_bytes(n, bits), oracle.num_blocks(n, B)
    err = torch.zeros(n, dtype=torch.float32, device=DEV)
    codes = torch.full((cb,), 0xAB, dtype=torch.uint8, device=DEV)
    scales = torch.full((nb,), 3.0, dtype=torch.bfloat16, device=DEV)
    ref_err = np.zeros(n, np.float32)
    for step in range(3):
        gt, gn = make_grad(rs, n, B, dtype)
        loco_compensate_quantize_bf16_scales(gt.to(DEV), err, bits, B, 0.25, False, codes, scales)
        torch.cuda.synchronize()
        rc, rscale = oracle.compensate_quantize(gn, ref_err, bits, B, 0.25, bf16_scales=True)
        assert np.array_equal(codes.cpu().numpy(), rc), step
        assert np.array_equal(u16(scales), rscale), step
        assert np.array_equal(err.cpu().numpy(), ref_err), step
    if n >= 4 * B:
        assert (rscale & 0x7F).any() and rscale[1] == 0 and rscale[2] == 0 and rscale[3] != 0


def test_step_just_under_flt_min_rounds_up_and_lives():
    n, B = 512, 256
    g = np.zeros(n, np.float32)
    g[0] = np.float32(7) * FLT_MIN * np.float32(1 - 2.0 ** -10)
    g[300] = np.float32(127) * FLT_MIN * np.float32(1 - 2.0 ** -10)
    for bits, hot in ((4, 0), (8, 300)):
        err = torch.zeros(n, dtype=torch.float32, device=DEV)
        codes = torch.zeros(oracle.code_bytes(n, bits), dtype=torch.uint8, device=DEV)
        scales = torch.zeros(2, dtype=torch.bfloat16, device=DEV)
        loco_compensate_quantize_bf16_scales(torch.from_numpy(g).to(DEV), err, bits, B, 1.0, False, codes, scales)
        torch.cuda.synchronize()
        ref_err = np.zeros(n, np.float32)
        rc, rscale = oracle.compensate_quantize(g, ref_err, bits, B, 1.0, bf16_scales=True)
        assert rscale[hot // B] == 0x0080
        assert np.array_equal(u16(scales), rscale) and np.array_equal(codes.cpu().numpy(), rc)
        assert np.array_equal(err.cpu().numpy(), ref_err)


@pytest.mark.parametrize("bits,B,W", [(4, 256, 8), (8, 64, 3), (4, 32, 1), (8, 512, 16), (4, 128, 5), (4, 64, 9)])
@pytest.mark.parametrize("n", [6 * 2048 + 777, 9, 2048])
def test_dequant_reduce_bf16_scales(bits, B, W, n):
    rs = np.random.default_rng(bits + B + W + n)
    cb, nb = oracle.code_bytes(n, bits), oracle.num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    sstride = nb + 3
    codes = rs.integers(0, 256, W * cstride, dtype=np.uint8)
    # any finite non-negative bf16 is a legal step: exponents over the whole range but the top
    # few binades (where W partial sums could overflow), some zeros
    top = 0xFA if W == 1 else 0xF0
    steps = ((rs.integers(1, top, W * sstride).astype(np.uint16) << 7) | rs.integers(0, 128, W * sstride).astype(np.uint16))
    steps[rs.random(W * sstride) < 0.1] = 0
    if 1 < W <= 9:      # a few steps of 2^120: 4-bit tiles that meet one are summed again without the 16*D shortcut
        steps[rs.random(W * sstride) < 0.02] = 0x7B80
    out = torch.full((n,), 7.0, dtype=torch.float32, device=DEV)
    st = torch.from_numpy(steps.view(np.int16)).view(torch.bfloat16).to(DEV)
    loco_dequant_reduce_bf16_scales(torch.from_numpy(codes).to(DEV), cstride, st, sstride, W, n, bits, B, out)
    torch.cuda.synchronize()
    want = oracle.dequant_reduce(codes, steps, W, n, bits, B, cstride, sstride)
    got = out.cpu().numpy()
    assert np.array_equal(got, want)
    assert np.isfinite(want).all() and np.any(want != 0)


def test_round_trip_single_worker_is_senders_decode():
    n, bits, B = 5 * 2048 + 100, 4, 256
    rs = np.random.default_rng(5)
    g = (rs.standard_normal(n) * 1e-3).astype(np.float32)
    err = torch.zeros(n, dtype=torch.float32, device=DEV)
    codes = torch.empty(oracle.code_bytes(n, bits), dtype=torch.uint8, device=DEV)
    scales = torch.empty(oracle.num_blocks(n, B), dtype=torch.bfloat16, device=DEV)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_compensate_quantize_bf16_scales(torch.from_numpy(g).to(DEV), err, bits, B, 1.0, False, codes, scales)
    loco_dequant_reduce_bf16_scales(codes, 0, scales, 0, 1, n, bits, B, out)
    torch.cuda.synchronize()
    d, delta = out.cpu().numpy(), err.cpu().numpy()      # beta = 1: the state is delta (Eq. 4)
    ref = oracle.dequant_reduce(codes.cpu().numpy(), u16(scales), 1, n, bits, B)
    assert np.array_equal(d, ref)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(d != 0, g.astype(np.float64) / d.astype(np.float64), 1.0)
    safe = (d == 0) | ((ratio >= 0.5) & (ratio <= 2.0))      # h - d exact there (Sterbenz)
    assert safe.mean() > 0.99
    assert np.array_equal((d + delta).astype(np.float32)[safe], g[safe])


def test_argument_errors():
    n, bits, B = 4096, 4, 256
    g = torch.zeros(n, dtype=torch.float32, device=DEV)
    err = torch.zeros(n, dtype=torch.float32, device=DEV)
    codes = torch.zeros(n // 2, dtype=torch.uint8, device=DEV)
    scales = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize_bf16_scales(g, err, 5, B, 0.25, False, codes, scales)
    assert ei.value.status == 2
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize_bf16_scales(g, err, bits, B, 1.5, False, codes, scales)
    assert ei.value.status == 1
    with pytest.raises(ValueError):
        loco_compensate_quantize_bf16_scales(g, err, bits, B, 0.25, False, codes, scales[:3])
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    with pytest.raises(LocoError) as ei:   # payload stride shorter than one payload
        loco_dequant_reduce_bf16_scales(torch.zeros(3 * n, dtype=torch.uint8, device=DEV), n // 2 - 16, scales, 16, 2, n,
                                        bits, B, out)
    assert ei.value.status == 1
