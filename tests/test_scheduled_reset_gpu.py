"""Eq. 7's reset schedule evaluated on the device (the _scheduled calls): the step index k
lives in device memory, the kernel zeroes the state when k % T_c == 0, so nothing about the
step is baked into a launch and ONE captured HIP graph of a step replays across reset steps.
Every step is compared with the oracle, whose own rule (oracle.reset_due) decides the flag."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize_fixed_f32state_scheduled,
                                  loco_compensate_quantize_fixed_scheduled, loco_compensate_quantize_scheduled,
                                  loco_error_state8_init, loco_error_state_init, loco_num_blocks,
                                  loco_step_index_advance, loco_step_index_set, workloads)
from paper_2407_04480_amd.binding import LocoError

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LOG2_S, SE_MULT = 19, 4


def fresh_gradient(n, dtype, seed):
    rng = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(n, generator=rng) * 1e-3).to(dtype)


@pytest.mark.parametrize("period,first", [(3, 0), (4, 0), (1, 5), (0, 0), (512, 510), ((1 << 33) + 1, 3 * ((1 << 33) + 1) - 2)])
@pytest.mark.parametrize("bits,B,dtype", [(4, 256, torch.bfloat16), (8, 64, torch.float32)])
def test_block_form_follows_the_schedule(period, first, bits, B, dtype):
    n = 5 * 2048 + 333
    k_dev = torch.zeros(1, dtype=torch.int64, device=DEV)
    loco_step_index_set(k_dev, first)
    err = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_error_state_init(err)
    e_ref = np.zeros(n, np.float32)
    codes = torch.zeros(loco_code_bytes(n, bits), dtype=torch.uint8, device=DEV)
    scales = torch.zeros(loco_num_blocks(n, B), dtype=torch.float32, device=DEV)
    resets = 0
    for j in range(2 * min(period, 4) + 3):
        k = first + j
        g = fresh_gradient(n, dtype, 100 + j)
        loco_compensate_quantize_scheduled(g.to(DEV), err, bits, B, 0.25, k_dev, period, codes, scales)
        loco_step_index_advance(k_dev)
        due = oracle.reset_due(k, period)
        resets += due
        c_ref, s_ref = oracle.compensate_quantize(workloads.as_numpy_grad(g), e_ref, bits, B, 0.25, int(due))
        torch.cuda.synchronize()
        assert int(k_dev.item()) == k + 1
        assert np.array_equal(codes.cpu().numpy(), c_ref), f"step {k}: codes"
        assert np.array_equal(scales.cpu().numpy().view(np.uint32), s_ref.view(np.uint32)), f"step {k}: steps"
        assert np.array_equal(err.cpu().numpy(), e_ref), f"step {k}: state"
        if due:
            assert not err.any()
    if period > 0 and period <= 4:
        assert resets >= 2
    if period == 0:
        assert resets == 0


def test_fixed_forms_follow_the_schedule():
    n, bits, T = 3 * 4096 + 77, 4, 3
    k_dev = torch.zeros(1, dtype=torch.int64, device=DEV)
    loco_step_index_set(k_dev, 0)
    e8 = torch.empty(n, dtype=torch.int8, device=DEV)
    loco_error_state8_init(e8)
    e32 = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_error_state_init(e32)
    e8_ref, e32_ref = np.zeros(n, np.int8), np.zeros(n, np.float32)
    c8 = torch.zeros(loco_code_bytes(n, bits), dtype=torch.uint8, device=DEV)
    c32 = torch.zeros_like(c8)
    for k in range(2 * T + 2):
        g = (fresh_gradient(n, torch.float32, 300 + k) * 4e-3).to(torch.bfloat16)
        loco_compensate_quantize_fixed_scheduled(g.to(DEV), e8, bits, LOG2_S, SE_MULT, 0.25, k_dev, T, c8)
        loco_compensate_quantize_fixed_f32state_scheduled(g.to(DEV), e32, bits, LOG2_S, 0.25, k_dev, T, c32)
        loco_step_index_advance(k_dev)
        due = int(oracle.reset_due(k, T))
        gh = workloads.as_numpy_grad(g)
        want8 = oracle.fixed_compensate_quantize(gh, e8_ref, bits, LOG2_S, SE_MULT, 0.25, due)
        want32 = oracle.fixed_compensate_quantize_f32state(gh, e32_ref, bits, LOG2_S, 0.25, due)
        torch.cuda.synchronize()
        assert np.array_equal(c8.cpu().numpy(), want8) and np.array_equal(e8.cpu().numpy(), e8_ref), f"step {k}"
        assert np.array_equal(c32.cpu().numpy(), want32) and np.array_equal(e32.cpu().numpy(), e32_ref), f"step {k}"
        assert bool(e8.any()) != bool(due) or due == 0


@pytest.mark.parametrize("form", ["block", "fixed"])
def test_one_captured_step_replays_across_reset_steps(form):
    """Capture [compensate-quantize (scheduled); advance k] ONCE and replay it 2 T_c + 1 times with
    T_c = 3: replays 0, 3 and 6 are reset steps although the graph never changes.  The gradient
    buffer the graph reads is refilled between replays by eager work on the host's side."""
    w = workloads.small("llama7b_shard_4bit_b256")
    n, bits, B, T = w.n, w.bits, w.block_size, 3
    g_buf = torch.zeros(n, dtype=w.grad_dtype, device=DEV)
    k_dev = torch.zeros(1, dtype=torch.int64, device=DEV)
    codes = torch.zeros(loco_code_bytes(n, bits), dtype=torch.uint8, device=DEV)
    scales = torch.zeros(loco_num_blocks(n, B), dtype=torch.float32, device=DEV)
    if form == "block":
        err = torch.empty(n, dtype=torch.float32, device=DEV)
        e_ref = np.zeros(n, np.float32)
        init = loco_error_state_init

        def step():
            loco_compensate_quantize_scheduled(g_buf, err, bits, B, w.beta, k_dev, T, codes, scales)
            loco_step_index_advance(k_dev)
    else:
        err = torch.empty(n, dtype=torch.int8, device=DEV)
        e_ref = np.zeros(n, np.int8)
        init = loco_error_state8_init

        def step():
            loco_compensate_quantize_fixed_scheduled(g_buf, err, bits, LOG2_S, SE_MULT, w.beta, k_dev, T, codes)
            loco_step_index_advance(k_dev)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        init(err)
        step()                          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    init(err)
    loco_step_index_set(k_dev, 0)
    torch.cuda.synchronize()
    seen_resets = 0
    for k in range(2 * T + 1):
        g = workloads.gradient(w, k)
        g_buf.copy_(g.to(DEV))          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        due = int(oracle.reset_due(k, T))
        seen_resets += due
        gh = workloads.as_numpy_grad(g)
        if form == "block":
            c_ref, s_ref = oracle.compensate_quantize(gh, e_ref, bits, B, w.beta, due)
            assert np.array_equal(scales.cpu().numpy().view(np.uint32), s_ref.view(np.uint32)), f"replay {k}: steps"
        else:
            c_ref = oracle.fixed_compensate_quantize(gh, e_ref, bits, LOG2_S, SE_MULT, w.beta, due)
        assert int(k_dev.item()) == k + 1
        assert np.array_equal(codes.cpu().numpy(), c_ref), f"replay {k}: codes"
        assert np.array_equal(err.cpu().numpy(), e_ref), f"replay {k}: state"
        assert bool(err.any()) == (not due), f"replay {k}: reset step {due} but state {'non-' if err.any() else ''}zero"
    assert seen_resets == 3


def test_scheduled_argument_errors():
    n = 1024
    g = torch.zeros(n, device=DEV)
    e = torch.zeros(n, device=DEV)
    c = torch.zeros(n // 2, dtype=torch.uint8, device=DEV)
    s = torch.zeros(n // 256, device=DEV)
    k = torch.zeros(2, dtype=torch.int64, device=DEV)
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize_scheduled(g, e, 4, 256, 0.25, k[:1], -1, c, s)
    assert ei.value.status == 1
    with pytest.raises(ValueError):
        loco_compensate_quantize_scheduled(g, e, 4, 256, 0.25, k, 3, c, s)
    with pytest.raises(TypeError):
        loco_compensate_quantize_scheduled(g, e, 4, 256, 0.25, torch.zeros(1, dtype=torch.int64), 3, c, s)
    odd = torch.zeros(3, dtype=torch.int32, device=DEV)[1:].view(torch.int32)   # 4 bytes past an 8-byte boundary
    from paper_2407_04480_amd import binding
    lib = binding.load_library()
    st = lib.loco_compensate_quantize_scheduled(g.data_ptr(), 0, e.data_ptr(), n, 4, 256, 0.25, odd.data_ptr(), 3,
                                                c.data_ptr(), s.data_ptr(), None)
    assert st == 3
