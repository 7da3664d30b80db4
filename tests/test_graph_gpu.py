"""The three calls under HIP graph capture: no call allocates, synchronises or records a
memset node (the state init is a fill kernel), so a training step can be captured once
and replayed.  Every replay is checked against the eager result, with eager work and
synchronisations between replays."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize, loco_dequant_reduce,
                                  loco_error_state_init, loco_num_blocks, workloads)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_step_replays_from_a_graph():
    w = workloads.gauss_1m()
    n, bits, B = w.n, w.bits, w.block_size
    cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B)
    g = workloads.gradient(w, 0, device=DEV)
    err = torch.empty(n, dtype=torch.float32, device=DEV)
    codes = torch.zeros(cb, dtype=torch.uint8, device=DEV)
    scales = torch.zeros(nb, dtype=torch.float32, device=DEV)
    out = torch.zeros(n, dtype=torch.float32, device=DEV)

    def one_step():
        loco_compensate_quantize(g, err, bits, B, w.beta, False, codes, scales)
        loco_dequant_reduce(codes, 0, scales, 0, 1, n, bits, B, out)

    # eager reference trajectory, and the oracle's, over 5 steps from a zero state
    loco_error_state_init(err)
    e_ref = np.zeros(n, np.float32)
    g_host = g.cpu().numpy()
    want = []
    for _ in range(5):
        one_step()
        torch.cuda.synchronize()
        c_ref, s_ref = oracle.compensate_quantize(g_host, e_ref, bits, B, w.beta)
        assert np.array_equal(codes.cpu().numpy(), c_ref) and np.array_equal(err.cpu().numpy(), e_ref)
        want.append((codes.clone(), scales.clone(), err.clone(), out.clone()))

    # capture: state init + one step in one graph, a bare step in another
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        loco_error_state_init(err)
        one_step()                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g_first, g_next = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_first):
        loco_error_state_init(err)
        one_step()
    with torch.cuda.graph(g_next):
        one_step()
    for round_ in range(3):
        g_first.replay()
        torch.cuda.synchronize()
        for k, (c, s, e, o) in enumerate(want):
            if k:
                g_next.replay()
                torch.cuda.synchronize()
            assert torch.equal(codes, c) and torch.equal(scales, s), f"round {round_} step {k}: payload"
            assert torch.equal(err, e) and torch.equal(out, o), f"round {round_} step {k}: state / output"
            # eager work between replays
            scratch = torch.randn(1 << 16, device=DEV).sum().item()
            assert np.isfinite(scratch)
