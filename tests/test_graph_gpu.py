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


def test_two_streams_overlap():
    """Compensate-quantize of the next bucket on one stream while the reduce of the previous
    bucket runs on another (the overlap the exchange would use): the calls share no state,
    so both streams' results equal the serial ones."""
    w = workloads.small("llama7b_shard_4bit_b256")
    n, bits, B, W = w.n, w.bits, w.block_size, 4
    cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B)
    cs = (cb + 15) // 16 * 16
    grads = [workloads.gradient(w, k, device=DEV) for k in range(W + 6)]

    def payloads(stream=None):
        codes = torch.zeros(W * cs, dtype=torch.uint8, device=DEV)
        scales = torch.zeros(W * nb, dtype=torch.float32, device=DEV)
        e = torch.empty(n, dtype=torch.float32, device=DEV)
        for k in range(W):
            loco_error_state_init(e, stream)
            loco_compensate_quantize(grads[k], e, bits, B, w.beta, False, codes[k * cs:k * cs + cb],
                                     scales[k * nb:(k + 1) * nb], stream)
        return codes, scales

    recv_codes, recv_scales = payloads()
    # serial reference: 6 steps of compensate-quantize, 6 reduces
    err = torch.zeros(n, dtype=torch.float32, device=DEV)
    oc, os_ = torch.zeros(cb, dtype=torch.uint8, device=DEV), torch.zeros(nb, dtype=torch.float32, device=DEV)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    serial = []
    for k in range(6):
        loco_compensate_quantize(grads[W + k], err, bits, B, w.beta, False, oc, os_)
        loco_dequant_reduce(recv_codes, cs, recv_scales, nb, W, n, bits, B, out)
        torch.cuda.synchronize()
        serial.append((oc.clone(), os_.clone(), err.clone(), out.clone()))
    # the same work with the two calls on two streams, no ordering between them
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    err.zero_()
    torch.cuda.synchronize()
    for k in range(6):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        loco_compensate_quantize(grads[W + k], err, bits, B, w.beta, False, oc, os_, a)
        loco_dequant_reduce(recv_codes, cs, recv_scales, nb, W, n, bits, B, out, b)
        a.synchronize()
        b.synchronize()
        c, s, e, o = serial[k]
        assert torch.equal(oc, c) and torch.equal(os_, s) and torch.equal(err, e), f"step {k}: compress"
        assert torch.equal(out, o), f"step {k}: reduce"
