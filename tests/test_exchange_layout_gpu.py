"""One LoCo step of N simulated ranks on ONE GPU, in the buffer layout an all-to-all would use.

Sec. 3.3 / App. A.1.4 of arXiv 2407.04480: every rank compresses its whole local gradient,
cuts the payload into N chunks, and an all-to-all hands chunk r of every rank to rank r, which
decodes and averages the N pieces it received (Eq. 8).  Here the N ranks are N sets of
buffers on the same device and the all-to-all is a strided device copy (no collective, no
second GPU); everything else is the library's calls exactly as a real rank would issue them:

  send buffer of rank s   N regions of `stride` bytes; region r = [codes of chunk r | its steps]
  receive buffer of rank r  region s = what rank s sent to r
  compress                one loco_compensate_quantize per chunk, writing straight into region r
  reduce                  one loco_dequant_reduce with code_stride = stride bytes and
                          scale_stride = stride/4 elements over the receive buffer

The oracle runs the same step on the host; payload bytes, states and averaged chunks must be
identical.  Lemma 1 averaged over the ranks (uncompressed state) is checked on the GPU's
results: sum_k g~_k = mean_s sum_k g^s_k - mean_s e~^s_K / beta.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_compensate_quantize, loco_dequant_reduce, loco_error_state_init, workloads)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("bits,B,ranks", [(4, 128, 4), (8, 64, 4), (4, 256, 8), (4, 32, 3)])
def test_simulated_ranks_all_to_all_layout(bits, B, ranks):
    N, K, beta = ranks, 5, 0.25
    chunk = 5 * 2048 + 3 * 256                      # elements per chunk: block aligned, ragged against the tiles
    psi = N * chunk                                 # local gradient of one rank
    cb = chunk * bits // 8                          # code bytes of one chunk
    nbk = chunk // B                                # blocks (steps) of one chunk
    assert chunk % B == 0 and cb % 16 == 0
    stride = (cb + 4 * nbk + 15) // 16 * 16         # one region: codes, then fp32 steps, padded to 16 bytes
    rng = torch.Generator(device="cpu").manual_seed(100 * bits + B + N)

    send = torch.zeros(N, N, stride, dtype=torch.uint8, device=DEV)       # [sender, destination, bytes]
    recv = torch.zeros(N, N, stride, dtype=torch.uint8, device=DEV)       # [receiver, source, bytes]
    err = torch.empty(N, psi, dtype=torch.float32, device=DEV)
    out = torch.empty(N, chunk, dtype=torch.float32, device=DEV)          # rank r ends with chunk r
    for s in range(N):
        loco_error_state_init(err[s])
    e_ref = np.zeros((N, psi), np.float32)
    send_ref = np.zeros((N, N, stride), np.uint8)
    sum_g = np.zeros((N, psi), np.float64)
    sum_avg = np.zeros((N, chunk), np.float64)
    scale_of_rank = [10.0 ** (-4 + s % 3) for s in range(N)]              # ranks see different magnitudes

    for k in range(K):
        grads = [(torch.randn(psi, generator=rng) * scale_of_rank[s]).to(torch.bfloat16) for s in range(N)]
        for s in range(N):
            g_dev = grads[s].to(DEV)
            g_host = workloads.as_numpy_grad(grads[s])
            sum_g[s] += grads[s].double().numpy()
            for r in range(N):                      # chunk r of rank s goes to rank r
                lo, hi = r * chunk, (r + 1) * chunk
                region = send[s, r]
                loco_compensate_quantize(g_dev[lo:hi], err[s, lo:hi], bits, B, beta, False,
                                         region[:cb], region[cb:cb + 4 * nbk].view(torch.float32))
                c_ref, s_ref = oracle.compensate_quantize(g_host[lo:hi], e_ref[s, lo:hi], bits, B, beta)
                send_ref[s, r, :cb] = c_ref
                send_ref[s, r, cb:cb + 4 * nbk] = s_ref.view(np.uint8)
        torch.cuda.synchronize()
        assert np.array_equal(send.cpu().numpy(), send_ref), f"step {k}: payload bytes differ"
        assert np.array_equal(err.cpu().numpy(), e_ref), f"step {k}: states differ"

        recv.copy_(send.transpose(0, 1))            # the all-to-all: region r of sender s -> region s of receiver r
        recv_ref = np.ascontiguousarray(send_ref.transpose(1, 0, 2))
        for r in range(N):
            flat = recv[r].reshape(-1)
            loco_dequant_reduce(flat, stride, flat[cb:].view(torch.float32), stride // 4, N, chunk, bits, B, out[r])
            flat_ref = recv_ref[r].reshape(-1)
            want = oracle.dequant_reduce(flat_ref, flat_ref[cb:].view(np.float32), N, chunk, bits, B, stride, stride // 4)
            torch.cuda.synchronize()
            got = out[r].cpu().numpy()
            assert np.array_equal(got, want), f"step {k} rank {r}: {np.count_nonzero(got != want)} averaged values differ"
            sum_avg[r] += got

    # Lemma 1 with an uncompressed state, averaged over the ranks, on the chunk each rank owns
    e_final = err.cpu().numpy().astype(np.float64)
    for r in range(N):
        lo, hi = r * chunk, (r + 1) * chunk
        want = sum_g[:, lo:hi].mean(axis=0) - e_final[:, lo:hi].mean(axis=0) / beta
        tol = K * 2.0 ** -20 * max(scale_of_rank) * 6
        assert np.abs(sum_avg[r] - want).max() <= tol
