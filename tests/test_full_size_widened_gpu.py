"""The widened entry points (clipping, bf16 block steps, bf16 output, reduce fused with the
optimizer steps of Eq. 9 / Eq. 10) on the 7B shard at FULL size, in the launch configuration
bench.py times.  As in test_full_size_gpu.py the oracle recomputes sampled blocks one by one
from the same input bytes; everything must match bit for bit.  Expected values come from the
oracle only."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize, loco_compensate_quantize_bf16_scales,
                                  loco_compensate_quantize_clip, loco_dequant_reduce_adam, loco_dequant_reduce_bf16,
                                  loco_dequant_reduce_bf16_scales, loco_dequant_reduce_sgd, loco_error_state_init,
                                  loco_num_blocks, workloads)
from test_full_size_gpu import code_index, element_index, host_grad, sample_blocks

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ETA, B1, B2, DL = 1e-4, 0.1, 0.02, 1e-8


def u16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def identical(name, got, want):
    assert got.shape == want.shape, name
    assert np.array_equal(got, want), f"{name}: {np.count_nonzero(got != want)} of {want.size} differ"


def test_full_size_widened_entry_points():
    w = workloads.by_name("llama7b_shard_4bit_b256")
    n, bits, B, W = w.n, w.bits, w.block_size, w.num_workers
    blocks = sample_blocks(w, count=2000, seed=23)
    eidx, cidx = element_index(blocks, B), code_index(blocks, B, bits)
    bidx = torch.from_numpy(blocks).to(DEV)
    ns = eidx.numel()
    cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    print(f"[widened] n={n} bits={bits} B={B} W={W} sampled blocks={blocks.size}", flush=True)

    err = torch.empty(n, dtype=torch.float32, device=DEV)
    codes = torch.zeros(W * cstride, dtype=torch.uint8, device=DEV)
    steps32 = torch.zeros(W * nb, dtype=torch.float32, device=DEV)
    steps16 = torch.zeros(W * nb + 1, dtype=torch.bfloat16, device=DEV)

    # ---- W payloads with bf16 steps (zero state each), the own one over two steps ----
    ref_codes = np.zeros((W, cidx.numel()), np.uint8)
    ref_steps = np.zeros((W, blocks.size), np.uint16)
    for k in range(W):
        loco_error_state_init(err)
        e_ref = np.zeros(ns, np.float32)
        for step in range(2 if k == 0 else 1):
            g = workloads.gradient(w, step, worker=k, device=DEV)
            loco_compensate_quantize_bf16_scales(g, err, bits, B, w.beta, False,
                                                 codes[k * cstride:k * cstride + cb], steps16[k * nb:(k + 1) * nb])
            ref_codes[k], ref_steps[k] = oracle.compensate_quantize(host_grad(g[eidx]), e_ref, bits, B, w.beta,
                                                                     bf16_scales=True)
            torch.cuda.synchronize()
            identical(f"bf16-step codes w={k} step={step}", codes[k * cstride:k * cstride + cb][cidx].cpu().numpy(),
                      ref_codes[k])
            identical(f"bf16 steps w={k} step={step}", u16(steps16[k * nb:(k + 1) * nb][bidx]), ref_steps[k])
            identical(f"state w={k} step={step}", err[eidx].cpu().numpy(), e_ref)
            del g
    assert int(steps16[W * nb:].view(torch.int16).item()) == 0          # nothing written past the last payload
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce_bf16_scales(codes, cstride, steps16, nb, W, n, bits, B, out)
    torch.cuda.synchronize()
    want = oracle.dequant_reduce(ref_codes.reshape(-1), ref_steps.reshape(-1), W, ns, bits, B,
                                 ref_codes.shape[1], ref_steps.shape[1])
    identical("bf16-step reduce", out[eidx].cpu().numpy(), want)
    assert bool(torch.isfinite(out).all())

    # ---- clipping: one step from a zero state; threshold at about the 90th percentile ----
    g = workloads.gradient(w, 0, device=DEV)
    g_s = host_grad(g[eidx])
    as_f32 = (g_s.astype(np.uint32) << 16).view(np.float32) if g_s.dtype == np.uint16 else g_s
    clip = float(np.quantile(np.abs(as_f32), 0.9))
    loco_error_state_init(err)
    loco_compensate_quantize_clip(g, clip, err, bits, B, w.beta, False, codes[:cb], steps32[:nb])
    e_ref = np.zeros(ns, np.float32)
    c_ref, s_ref = oracle.compensate_quantize(oracle.clip_gradient(g_s, clip), e_ref, bits, B, w.beta)
    torch.cuda.synchronize()
    identical("clip codes", codes[:cb][cidx].cpu().numpy(), c_ref)
    identical("clip steps", steps32[:nb][bidx].cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    identical("clip state", err[eidx].cpu().numpy(), e_ref)
    assert float(s_ref.max()) * 7 <= clip * (1 + 1e-6) and bool((np.abs(as_f32) > clip).any())
    del g

    # ---- W fp32-step payloads for the reduce epilogues ----
    ref_steps32 = np.zeros((W, blocks.size), np.float32)
    for k in range(W):
        g = workloads.gradient(w, 0, worker=k, device=DEV)
        loco_error_state_init(err)
        loco_compensate_quantize(g, err, bits, B, w.beta, False, codes[k * cstride:k * cstride + cb],
                                 steps32[k * nb:(k + 1) * nb])
        ref_codes[k], ref_steps32[k] = oracle.compensate_quantize(host_grad(g[eidx]), np.zeros(ns, np.float32),
                                                                   bits, B, w.beta)
        del g
    torch.cuda.synchronize()
    g_avg = oracle.dequant_reduce(ref_codes.reshape(-1), ref_steps32.reshape(-1), W, ns, bits, B,
                                  ref_codes.shape[1], ref_steps32.shape[1])
    del err

    out16 = torch.full((n,), float("nan"), dtype=torch.bfloat16, device=DEV)
    loco_dequant_reduce_bf16(codes, cstride, steps32, nb, W, n, bits, B, out16)
    torch.cuda.synchronize()
    identical("bf16 output", u16(out16[eidx]), oracle.round_to_bf16(g_avg))
    assert bool(torch.isfinite(out16).all())
    del out16

    theta = torch.empty(n, dtype=torch.float32, device=DEV)
    theta.normal_(generator=torch.Generator(device=DEV).manual_seed(7))
    th_sgd_h = theta[eidx].cpu().numpy().copy()
    th_adam_h = th_sgd_h.copy()
    loco_dequant_reduce_sgd(codes, cstride, steps32, nb, W, n, bits, B, ETA, theta)
    torch.cuda.synchronize()
    oracle.sgd_update(th_sgd_h, g_avg, ETA)
    identical("sgd theta", theta[eidx].cpu().numpy(), th_sgd_h)

    theta[eidx] = torch.from_numpy(th_adam_h).to(DEV)          # same starting point on the sample
    mom, var = torch.zeros_like(theta), torch.zeros_like(theta)
    m_h, v_h = np.zeros(ns, np.float32), np.zeros(ns, np.float32)
    for step in range(2):
        loco_dequant_reduce_adam(codes, cstride, steps32, nb, W, n, bits, B, ETA, B1, B2, DL, mom, var, theta)
        torch.cuda.synchronize()
        oracle.adam_update(th_adam_h, m_h, v_h, g_avg, ETA, B1, B2, DL)
        identical(f"adam m step {step}", mom[eidx].cpu().numpy(), m_h)
        identical(f"adam v step {step}", var[eidx].cpu().numpy(), v_h)
        identical(f"adam theta step {step}", theta[eidx].cpu().numpy(), th_adam_h)
    assert bool(torch.isfinite(theta).all()) and bool((var >= 0).all())
