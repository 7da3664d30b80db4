"""Compensate-quantize at lengths around the boundaries of its tile order.

The compressor hands its tiles to the XCDs in runs of 32768 consecutive elements, eight runs
(262144 elements) per round of workgroups, and rounds its grid up to whole rounds.  Alg. 1
steps 1-2 do not care which workgroup takes which tile: every element must be produced exactly
once, whatever part of the last round is empty.  Lengths just below, at and just above whole
runs and whole rounds, for both workgroup sizes of the block form (4- and 8-bit codes) and for
the fixed-scale form with the state in float32, against the oracle byte for byte.  With the
canaries behind every output this also shows that the empty tiles of the last round write nothing.

The runs are laid over the state's ADDRESSES (each starts at a multiple of 128 KB), so as many
tile indices as the state's first byte lies behind such a multiple stay empty in front: the
test after those moves the state through offsets of 16 bytes to 128 KB within its allocation.
The reduces (Alg. 1 step 3, Eq. 8) lay their runs over the array they write or update in place
in the same way; the last tests move that array, for every launch shape the worker count selects.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize,
                                  loco_compensate_quantize_fixed_f32state, loco_dequant_reduce, loco_dequant_reduce_adam,
                                  loco_dequant_reduce_bf16, loco_dequant_reduce_fixed, loco_dequant_reduce_fixed_adam,
                                  loco_dequant_reduce_fixed_bf16, loco_dequant_reduce_sgd, loco_num_blocks, workloads)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RUN, ROUND = 32768, 8 * 32768
LENGTHS = [RUN - 1, RUN, RUN + 1, 3 * RUN + 1024 + 5, ROUND - 1, ROUND, ROUND + 1, ROUND + RUN + 1,
           2 * ROUND + 5 * RUN - 3, 5 * ROUND - 2048]
PAD = 64   # canary elements behind every output


def gradient(n, dtype, seed):
    rng = torch.Generator(device="cpu").manual_seed(seed)
    g = torch.randn(n, generator=rng) * 1e-3
    g[:: 4099] *= 50.0              # a few blocks with a large step
    g[7 * 256: 9 * 256] = 0.0       # two dead blocks
    return g.to(dtype)


@pytest.mark.parametrize("bits,B", [(4, 256), (4, 32), (8, 64), (8, 512)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_block_form_around_run_and_round_boundaries(bits, B, dtype):
    for n in LENGTHS:
        print(f"[tile order] block form bits={bits} B={B} {dtype} n={n}", flush=True)
        cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B)
        e_host = np.zeros(n, np.float32)
        e_t = torch.full((n + PAD,), 5.0, dtype=torch.float32, device=DEV)
        e_t[:n] = 0.0
        codes_t = torch.full((cb + PAD,), 0xAA, dtype=torch.uint8, device=DEV)
        scales_t = torch.full((nb + PAD,), -1.0, dtype=torch.float32, device=DEV)
        for step in range(2):
            g = gradient(n, dtype, 31 * n + step)
            loco_compensate_quantize(g.to(DEV), e_t[:n], bits, B, 0.25, False, codes_t[:cb], scales_t[:nb])
            torch.cuda.synchronize()
            c_ref, s_ref = oracle.compensate_quantize(workloads.as_numpy_grad(g), e_host, bits, B, 0.25, 0)
            assert np.array_equal(codes_t[:cb].cpu().numpy(), c_ref), f"n={n} step={step}: code bytes differ"
            assert np.array_equal(scales_t[:nb].cpu().numpy().view(np.uint32), s_ref.view(np.uint32)), f"n={n}: steps differ"
            assert np.array_equal(e_t[:n].cpu().numpy(), e_host), f"n={n} step={step}: state differs"
        assert bool((e_t[n:] == 5.0).all()) and bool((codes_t[cb:] == 0xAA).all()) and bool((scales_t[nb:] == -1.0).all()), \
            f"n={n}: written past the end"


@pytest.mark.parametrize("bits", [4, 8])
def test_fixed_scale_form_with_fp32_state_around_run_and_round_boundaries(bits):
    log2_s = 19 if bits == 4 else 17
    for n in LENGTHS:
        print(f"[tile order] fixed scale, fp32 state, bits={bits} n={n}", flush=True)
        cb = loco_code_bytes(n, bits)
        e_host = np.zeros(n, np.float32)
        e_t = torch.full((n + PAD,), 5.0, dtype=torch.float32, device=DEV)
        e_t[:n] = 0.0
        codes_t = torch.full((cb + PAD,), 0xAA, dtype=torch.uint8, device=DEV)
        for step in range(2):
            g = (gradient(n, torch.bfloat16, 17 * n + step).float() * 1e-2).to(torch.bfloat16)
            loco_compensate_quantize_fixed_f32state(g.to(DEV), e_t[:n], bits, log2_s, 0.25, False, codes_t[:cb])
            torch.cuda.synchronize()
            c_ref = oracle.fixed_compensate_quantize_f32state(workloads.as_numpy_grad(g), e_host, bits, log2_s, 0.25)
            assert np.array_equal(codes_t[:cb].cpu().numpy(), c_ref), f"n={n} step={step}: code bytes differ"
            assert np.array_equal(e_t[:n].cpu().numpy(), e_host), f"n={n} step={step}: state differs"
        assert bool((e_t[n:] == 5.0).all()) and bool((codes_t[cb:] == 0xAA).all()), f"n={n}: written past the end"


# elements in front of the state inside its allocation (16-byte steps; a tile is 512 elements, a run 32768)
STATE_OFFSETS = [4, 508, 512, 516, 3 * 512 + 8, 16384 + 4, 32768 - 4, 32768, 32768 + 512]


@pytest.mark.parametrize("form,bits,B", [("block", 4, 256), ("block", 8, 64), ("block", 4, 32), ("fixed_f32", 4, 0), ("fixed_f32", 8, 0)])
def test_state_at_any_16_byte_offset(form, bits, B):
    for off in STATE_OFFSETS:
        for n in (RUN - off % RUN + 5, ROUND + 3 * RUN - 2048 + 1, 2 * ROUND - off):
            print(f"[tile order] {form} bits={bits} B={B} state offset {off} elements, n={n}", flush=True)
            cb = loco_code_bytes(n, bits)
            nb = loco_num_blocks(n, B) if form == "block" else 0
            e_host = np.zeros(n, np.float32)
            e_all = torch.full((off + n + PAD,), 5.0, dtype=torch.float32, device=DEV)
            e_t = e_all[off:off + n]
            e_t.zero_()
            codes_t = torch.full((cb + PAD,), 0xAA, dtype=torch.uint8, device=DEV)
            scales_t = torch.full((nb + PAD,), -1.0, dtype=torch.float32, device=DEV)
            for step in range(2):
                if form == "block":
                    g = gradient(n, torch.bfloat16, 13 * n + off + step)
                    loco_compensate_quantize(g.to(DEV), e_t, bits, B, 0.25, False, codes_t[:cb], scales_t[:nb])
                    torch.cuda.synchronize()
                    c_ref, s_ref = oracle.compensate_quantize(workloads.as_numpy_grad(g), e_host, bits, B, 0.25, 0)
                    assert np.array_equal(scales_t[:nb].cpu().numpy().view(np.uint32), s_ref.view(np.uint32)), f"off={off} n={n}: steps differ"
                else:
                    g = (gradient(n, torch.bfloat16, 13 * n + off + step).float() * 1e-2).to(torch.bfloat16)
                    loco_compensate_quantize_fixed_f32state(g.to(DEV), e_t, bits, 19 if bits == 4 else 17, 0.25, False, codes_t[:cb])
                    torch.cuda.synchronize()
                    c_ref = oracle.fixed_compensate_quantize_f32state(workloads.as_numpy_grad(g), e_host, bits, 19 if bits == 4 else 17, 0.25)
                assert np.array_equal(codes_t[:cb].cpu().numpy(), c_ref), f"off={off} n={n} step={step}: code bytes differ"
                assert np.array_equal(e_t.cpu().numpy(), e_host), f"off={off} n={n} step={step}: state differs"
            assert bool((e_all[:off] == 5.0).all()) and bool((e_all[off + n:] == 5.0).all()), f"off={off} n={n}: state written outside"
            assert bool((codes_t[cb:] == 0xAA).all()) and bool((scales_t[nb:] == -1.0).all()), f"off={off} n={n}: written past the end"


def reduce_inputs(n, bits, B, W, seed):
    rs = np.random.default_rng(seed)
    cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B) if B else 0
    cs, ss = (cb + 15) // 16 * 16 + 48, nb + 3
    codes = rs.integers(0, 256, W * cs, dtype=np.uint8)
    scales = (rs.uniform(0.5, 2.0, W * ss) * 1e-4).astype(np.float32) if B else None
    return codes, scales, cs, ss


# output elements in front of the output inside its allocation (16-byte steps of fp32, and of bf16)
OUT_OFFSETS = [4, 1020, 1024, 2 * 1024 + 8, 16384 + 12, 32768 - 4, 65536 + 2048]


@pytest.mark.parametrize("bits,B,W", [(4, 256, 1), (4, 128, 2), (8, 64, 1), (8, 64, 3), (4, 256, 8), (8, 64, 8), (4, 64, 16),
                                      (4, 256, 70), (8, 256, 9), (4, 32, 5)])
def test_reduce_output_at_any_16_byte_offset(bits, B, W):
    n = (ROUND + 3 * RUN + 1024 + 7) if W <= 16 else (1 << 22) + 2048 + 5
    codes, scales, cs, ss = reduce_inputs(n, bits, B, W, 100 * W + bits)
    want = oracle.dequant_reduce(codes, scales, W, n, bits, B, cs, ss, threads=8)
    want_bf16 = oracle.round_to_bf16(want)
    c_t, s_t = torch.from_numpy(codes).to(DEV), torch.from_numpy(scales).to(DEV)
    for off in OUT_OFFSETS:
        print(f"[tile order] reduce bits={bits} B={B} W={W} n={n}, output offset {off} elements", flush=True)
        out_all = torch.full((off + n + PAD,), 5.0, dtype=torch.float32, device=DEV)
        loco_dequant_reduce(c_t, cs, s_t, ss, W, n, bits, B, out_all[off:off + n])
        torch.cuda.synchronize()
        assert np.array_equal(out_all[off:off + n].cpu().numpy(), want), f"off={off}: averaged gradient differs"
        assert bool((out_all[:off] == 5.0).all()) and bool((out_all[off + n:] == 5.0).all()), f"off={off}: written outside"
        o16_all = torch.full((2 * off + n + PAD,), 5.0, dtype=torch.bfloat16, device=DEV)
        loco_dequant_reduce_bf16(c_t, cs, s_t, ss, W, n, bits, B, o16_all[2 * off:2 * off + n])
        torch.cuda.synchronize()
        got = o16_all[2 * off:2 * off + n].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want_bf16), f"off={off}: bf16 output differs"
        assert bool((o16_all[:2 * off] == 5.0).all()) and bool((o16_all[2 * off + n:] == 5.0).all()), f"off={off}: bf16 written outside"


@pytest.mark.parametrize("bits,W", [(4, 1), (4, 3), (8, 1), (4, 8), (8, 8), (4, 40)])
def test_fixed_reduce_output_at_any_16_byte_offset(bits, W):
    n = ROUND + 3 * RUN + 1024 + 7
    codes, _, cs, _ = reduce_inputs(n, bits, 0, W, 200 * W + bits)
    want = oracle.fixed_dequant_reduce(codes, W, n, bits, 19, code_stride_bytes=cs)
    want_bf16 = oracle.round_to_bf16(want)
    c_t = torch.from_numpy(codes).to(DEV)
    for off in OUT_OFFSETS:
        print(f"[tile order] fixed reduce bits={bits} W={W} n={n}, output offset {off} elements", flush=True)
        out_all = torch.full((off + n + PAD,), 5.0, dtype=torch.float32, device=DEV)
        loco_dequant_reduce_fixed(c_t, cs, W, n, bits, 19, out_all[off:off + n])
        torch.cuda.synchronize()
        assert np.array_equal(out_all[off:off + n].cpu().numpy(), want), f"off={off}: averaged gradient differs"
        assert bool((out_all[:off] == 5.0).all()) and bool((out_all[off + n:] == 5.0).all()), f"off={off}: written outside"
        o16_all = torch.full((2 * off + n + PAD,), 5.0, dtype=torch.bfloat16, device=DEV)
        loco_dequant_reduce_fixed_bf16(c_t, cs, W, n, bits, 19, o16_all[2 * off:2 * off + n])
        torch.cuda.synchronize()
        got = o16_all[2 * off:2 * off + n].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want_bf16), f"off={off}: bf16 output differs"
        assert bool((o16_all[:2 * off] == 5.0).all()) and bool((o16_all[2 * off + n:] == 5.0).all()), f"off={off}: bf16 written outside"


@pytest.mark.parametrize("bits,B,W", [(4, 256, 8), (8, 64, 2), (4, 256, 70)])
def test_fused_optimizers_with_parameters_at_any_16_byte_offset(bits, B, W):
    eta, b1, b2, dl = 1e-3, 0.9, 0.999, 1e-8
    n = (ROUND + 3 * RUN + 1024 + 7) if W <= 16 else (1 << 22) + 2048 + 5
    codes, scales, cs, ss = reduce_inputs(n, bits, B, W, 300 * W + bits)
    g_avg = oracle.dequant_reduce(codes, scales, W, n, bits, B, cs, ss, threads=8)
    g_fix = oracle.fixed_dequant_reduce(codes, W, n, bits, 19, code_stride_bytes=cs)
    th0 = np.random.default_rng(5).standard_normal(n).astype(np.float32)
    want = {}
    for name, g in (("block", g_avg), ("fixed", g_fix)):
        th_s, th_a, m, v = th0.copy(), th0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
        oracle.sgd_update(th_s, g, eta)
        oracle.adam_update(th_a, m, v, g, eta, b1, b2, dl)
        want[name] = (th_s, th_a, m, v)
    c_t, s_t = torch.from_numpy(codes).to(DEV), torch.from_numpy(scales).to(DEV)
    for off in OUT_OFFSETS[1::2]:
        for name in ("block", "fixed"):
            print(f"[tile order] {name} reduce + optimizer bits={bits} B={B} W={W}, parameters offset {off} elements", flush=True)
            arrays = [torch.full((off + n + PAD,), 5.0, dtype=torch.float32, device=DEV) for _ in range(4)]
            th_s, th_a, m, v = (a[off:off + n] for a in arrays)
            th_s.copy_(torch.from_numpy(th0)); th_a.copy_(torch.from_numpy(th0)); m.zero_(); v.zero_()
            if name == "block":
                loco_dequant_reduce_sgd(c_t, cs, s_t, ss, W, n, bits, B, eta, th_s)
                loco_dequant_reduce_adam(c_t, cs, s_t, ss, W, n, bits, B, eta, b1, b2, dl, m, v, th_a)
            else:
                from paper_2407_04480_amd import loco_dequant_reduce_fixed_sgd
                loco_dequant_reduce_fixed_sgd(c_t, cs, W, n, bits, 19, eta, th_s)
                loco_dequant_reduce_fixed_adam(c_t, cs, W, n, bits, 19, eta, b1, b2, dl, m, v, th_a)
            torch.cuda.synchronize()
            for what, got, ref in zip(("sgd theta", "adam theta", "m", "v"), (th_s, th_a, m, v), want[name]):
                assert np.array_equal(got.cpu().numpy(), ref), f"{name} off={off}: {what} differs"
            for a in arrays:
                assert bool((a[:off] == 5.0).all()) and bool((a[off + n:] == 5.0).all()), f"{name} off={off}: written outside"
