"""The benchmark workloads at FULL size, through the same C-ABI calls (hence the same
launch configuration) that bench.py times.

The oracle cannot sweep 10^9 elements for every step of every test in seconds, but
blocks are independent (compensate-quantize) and elements are independent (dequant-
reduce), so it recomputes SAMPLED blocks one by one, step by step, from the same input
bytes: the first and last blocks, the blocks on both sides of every tensor boundary and
a few thousand at random.  They must match bit for bit (codes, steps) and within 1e-6
(state, averaged gradient; in fact identically).  Whole-array properties that hold at
any size are checked with device-side reductions.  Expected values come from the oracle
only; the GPU's payloads are never fed to it.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize, loco_dequant_reduce,
                                  loco_error_state_init, loco_num_blocks, workloads)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FULL = ["llama7b_shard_4bit_b256", "llama7b_shard_8bit_b64", "mixtral_moe_shard_4bit_b128",
        "dense70b_shard_4bit_b256"]
# every step of every workload: 20 for the dense shards, 10 for the MoE shard (error accumulation)
STEPS = {"llama7b_shard_4bit_b256": 20, "llama7b_shard_8bit_b64": 20, "mixtral_moe_shard_4bit_b128": 10,
         "dense70b_shard_4bit_b256": 20}


def sample_blocks(w: workloads.Workload, count=3000, seed=11):
    nb = w.n // w.block_size
    rs = np.random.default_rng(seed)
    picks = set(rs.integers(0, nb, count).tolist())
    picks.update(range(0, 4))
    picks.update(range(nb - 4, nb))
    for _, start, length in w.segments:        # both sides of every tensor boundary
        for edge in (start, start + length):
            b = edge // w.block_size
            for d in (-1, 0, 1):
                if 0 <= b + d < nb:
                    picks.add(b + d)
    # tile edges of the kernels (512-element wavefront tiles, 1024..2048-element workgroups)
    for t in rs.integers(1, w.n // 2048, 64):
        b = int(t) * 2048 // w.block_size
        picks.update({b - 1, b})
    return np.array(sorted(picks), dtype=np.int64)


def element_index(blocks: np.ndarray, B: int) -> torch.Tensor:
    idx = (blocks[:, None] * B + np.arange(B)[None, :]).reshape(-1)
    return torch.from_numpy(idx).to(DEV)


def code_index(blocks: np.ndarray, B: int, bits: int) -> torch.Tensor:
    per = B * bits // 8
    idx = (blocks[:, None] * per + np.arange(per)[None, :]).reshape(-1)
    return torch.from_numpy(idx).to(DEV)


def host_grad(t: torch.Tensor):
    return workloads.as_numpy_grad(t)


@pytest.mark.parametrize("name", FULL)
def test_full_size_against_sampled_oracle(name):
    w = workloads.by_name(name)
    n, bits, B, W = w.n, w.bits, w.block_size, w.num_workers
    assert n % B == 0 and n % 2 == 0
    blocks = sample_blocks(w)
    eidx, cidx = element_index(blocks, B), code_index(blocks, B, bits)
    bidx = torch.from_numpy(blocks).to(DEV)
    ns = eidx.numel()
    cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    print(f"[{name}] n={n} bits={bits} B={B} W={W} sampled blocks={blocks.size}", flush=True)

    err = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_error_state_init(err)
    recv_codes = torch.zeros(W * cstride, dtype=torch.uint8, device=DEV)
    recv_scales = torch.zeros(W * nb, dtype=torch.float32, device=DEV)
    own_codes, own_scales = recv_codes[:cb], recv_scales[:nb]
    grads = [workloads.gradient(w, s, device=DEV) for s in range(2)]   # ring of two, as in bench.py
    e_ref = np.zeros(ns, np.float32)
    qmax = (1 << (bits - 1)) - 1
    # Lemma 1 telescoped over the steps, on the GPU's own outputs, accumulated in float64 on the device
    decoded = torch.empty(n, dtype=torch.float32, device=DEV)
    sum_d = torch.zeros(ns, dtype=torch.float64, device=DEV)
    sum_g = torch.zeros(ns, dtype=torch.float64, device=DEV)
    step_max = torch.zeros(blocks.size, dtype=torch.float32, device=DEV)

    for step in range(STEPS[name]):
        g = grads[step & 1]
        g_s = host_grad(g[eidx])
        loco_compensate_quantize(g, err, bits, B, w.beta, False, own_codes, own_scales)
        loco_dequant_reduce(own_codes, 0, own_scales, 0, 1, n, bits, B, decoded)      # d_k, what a receiver decodes
        sum_d += decoded[eidx].double()
        sum_g += g[eidx].double()
        step_max = torch.maximum(step_max, own_scales[bidx])
        c_ref, s_ref = oracle.compensate_quantize(g_s, e_ref, bits, B, w.beta)
        torch.cuda.synchronize()
        c_gpu = own_codes[cidx].cpu().numpy()
        s_gpu = own_scales[bidx].cpu().numpy()
        e_gpu = err[eidx].cpu().numpy()
        assert np.array_equal(c_gpu, c_ref), f"step {step}: {np.count_nonzero(c_gpu != c_ref)} code bytes differ"
        assert np.array_equal(s_gpu.view(np.uint32), s_ref.view(np.uint32)), f"step {step}: steps differ"
        top = float(np.abs(e_ref).max())
        assert float(np.abs(e_gpu.astype(np.float64) - e_ref).max()) <= 1e-6 * top
        assert np.count_nonzero(e_gpu != e_ref) == 0, f"step {step}: state not identical"

    # ---- Lemma 1 with an uncompressed state, telescoped: sum_k d_k = sum_k g_k - e~_K / beta ----
    # Per step the binary32 roundings of h = g + e~ and of the fmaf of Eq. 5 enter the identity with at
    # most 2^-24 (|h| + |e~'| / beta) <= 2^-24 D (qmax + 1 / (2 beta)); the bound below doubles that.
    K = STEPS[name]
    residual = (sum_d - (sum_g - err[eidx].double() / w.beta)).abs().view(blocks.size, B).amax(dim=1)
    bound = K * 2.0 ** -24 * 2.0 * (qmax + 0.5 / w.beta) * step_max.double()
    worst = float((residual / bound.clamp_min(1e-300)).max())
    assert bool((residual <= bound).all()), f"Lemma 1 after {K} steps: residual up to {worst:.3f} of the bound"
    assert bool((residual[step_max == 0] == 0).all())
    print(f"[{name}] Lemma 1 telescoped over {K} steps: largest residual {worst:.3f} of the rounding bound", flush=True)
    del decoded, sum_d, sum_g

    # ---- whole-array properties of the last payload (device-side reductions) ----
    scales_all = own_scales
    assert bool(torch.isfinite(scales_all).all()) and bool((scales_all >= 0).all())
    if bits == 8:
        q = own_codes.view(torch.int8).view(nb, B)
        assert int((q == -128).sum()) == 0                       # the clamp never fires
        amax = q.abs().amax(dim=1)
    else:
        lo = (own_codes & 15).view(nb, B // 2)
        hi = (own_codes >> 4).view(nb, B // 2)
        assert int((lo == 8).sum()) == 0 and int((hi == 8).sum()) == 0
        mag = lambda x: torch.where(x >= 8, 16 - x.to(torch.int16), x.to(torch.int16))
        amax = torch.maximum(mag(lo).amax(dim=1), mag(hi).amax(dim=1))
        del lo, hi
    live = scales_all > 0
    assert bool((amax[live] == qmax).all()), "a live block without a +-qmax code"
    assert bool((amax[~live] == 0).all()), "a dead block with non-zero codes"
    if w.recipe == "moe":                                       # unrouted experts stay exactly zero
        for e_id in workloads.ZERO_EXPERTS:
            _, start, length = w.segments[e_id]
            assert not bool(scales_all[start // B:(start + length) // B].any())
            assert not bool(err[start:start + length].any())
            assert not bool(own_codes[start * bits // 8:(start + length) * bits // 8].any())
    del amax, live

    # ---- dequant-reduce over W payloads: slot 0 is this worker's last payload ----
    tmp = torch.empty(n, dtype=torch.float32, device=DEV)
    ref_codes = np.zeros((W, cidx.numel()), np.uint8)
    ref_scales = np.zeros((W, blocks.size), np.float32)
    ref_codes[0], ref_scales[0] = c_ref, s_ref
    for k in range(1, W):
        gk = workloads.gradient(w, 0, worker=k, device=DEV)
        loco_error_state_init(tmp)
        loco_compensate_quantize(gk, tmp, bits, B, w.beta, False,
                                 recv_codes[k * cstride:k * cstride + cb], recv_scales[k * nb:(k + 1) * nb])
        ref_codes[k], ref_scales[k] = oracle.compensate_quantize(host_grad(gk[eidx]), np.zeros(ns, np.float32),
                                                                  bits, B, w.beta)
        torch.cuda.synchronize()
        assert np.array_equal(recv_codes[k * cstride:k * cstride + cb][cidx].cpu().numpy(), ref_codes[k])
        del gk
    del tmp
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out)
    torch.cuda.synchronize()
    want = oracle.dequant_reduce(ref_codes.reshape(-1), ref_scales.reshape(-1), W, ns, bits, B,
                                 ref_codes.shape[1], ref_scales.shape[1])
    got = out[eidx].cpu().numpy()
    assert float(np.abs(got.astype(np.float64) - want).max()) <= 1e-6 * float(np.abs(want).max())
    assert np.count_nonzero(got != want) == 0, "averaged gradient not identical on the sampled blocks"
    assert bool(torch.isfinite(out).all())        # every element was written over the NaN fill


def test_full_size_exact_reconstruction():
    """Eq. 4 at full size and through both kernels: with beta = 1 the new state is h - d,
    and dequant-reduce with N = 1 returns d, so d + state gives back the gradient exactly
    (a zero initial state makes h = g)."""
    w = workloads.by_name("llama7b_shard_4bit_b256")
    n, bits, B = w.n, w.bits, w.block_size
    g = workloads.gradient(w, 0, device=DEV)
    err = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_error_state_init(err)
    codes = torch.empty(loco_code_bytes(n, bits), dtype=torch.uint8, device=DEV)
    scales = torch.empty(loco_num_blocks(n, B), dtype=torch.float32, device=DEV)
    loco_compensate_quantize(g, err, bits, B, 1.0, False, codes, scales)
    d = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_dequant_reduce(codes, 0, scales, 0, 1, n, bits, B, d)
    torch.cuda.synchronize()
    d += err
    g32 = g.float()
    mism = d != g32
    bad = int(mism.sum())
    assert bad <= 1e-4 * n, f"{bad} of {n} elements do not reconstruct exactly"
    if bad:
        # the remaining cases are |q| = 1 with |h| a hair under half a step: off by one rounding
        rel = ((d - g32).abs()[mism] / g32.abs()[mism]).max()
        assert float(rel) <= 2.0 ** -22
    # Lemma 5: |h - d| <= D/2 (+ rounding of 1/D), for every element
    step = scales.repeat_interleave(B)[:n]
    assert bool((err.abs() <= step * (0.5 + 2.0 ** -18)).all())


@pytest.mark.parametrize("name,steps", [("llama7b_shard_4bit_b256", 2), ("llama7b_shard_8bit_b64", 2),
                                        ("mixtral_moe_shard_4bit_b128", 3), ("dense70b_shard_4bit_b256", 1)])
def test_full_size_every_element(name, steps, capsys):
    """A workload compared with the oracle over the WHOLE array, not a sample: a few steps of
    compensate-quantize (every code byte, every block step, every state value) and the reduce
    over the W payloads (every element of the averaged gradient; the largest workload has more
    than 2^31 elements and 16 payloads).  The oracle runs on all host threads over disjoint
    block ranges, which gives the bytes of its single-threaded run."""
    import os

    def print(*a, **k):   # progress lines reach the terminal also when pytest captures output
        import builtins
        with capsys.disabled():
            builtins.print(*a, **k)

    w = workloads.by_name(name)
    n, bits, B, W = w.n, w.bits, w.block_size, w.num_workers
    threads = max(1, min(16, os.cpu_count() or 1))
    cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    print(f"[{name}] whole array: n={n} bits={bits} B={B} W={W} oracle threads={threads}", flush=True)
    err = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_error_state_init(err)
    recv_codes = torch.zeros(W * cstride, dtype=torch.uint8, device=DEV)
    recv_scales = torch.zeros(W * nb, dtype=torch.float32, device=DEV)
    e_ref = np.zeros(n, np.float32)
    ref_codes = np.zeros((W, cstride), np.uint8)
    ref_scales = np.zeros((W, nb), np.float32)
    for step in range(steps):
        g = workloads.gradient(w, step, device=DEV)
        loco_compensate_quantize(g, err, bits, B, w.beta, False, recv_codes[:cb], recv_scales[:nb])
        c_ref, s_ref = oracle.compensate_quantize(host_grad(g), e_ref, bits, B, w.beta, threads=threads)
        torch.cuda.synchronize()
        del g
        assert np.array_equal(recv_codes[:cb].cpu().numpy(), c_ref), f"step {step}: code bytes differ"
        assert np.array_equal(recv_scales[:nb].cpu().numpy().view(np.uint32), s_ref.view(np.uint32)), \
            f"step {step}: block steps differ"
        e_gpu = err.cpu().numpy()
        bad = int(np.count_nonzero(e_gpu != e_ref))
        assert bad == 0, f"step {step}: {bad} of {n} state values differ"
        del e_gpu
        print(f"[{name}] step {step}: codes, steps and state identical over {n} elements", flush=True)
    ref_codes[0, :cb], ref_scales[0] = c_ref, s_ref
    del c_ref, s_ref, e_ref
    tmp = torch.empty(n, dtype=torch.float32, device=DEV)
    zero = np.zeros(n, np.float32)
    for k in range(1, W):
        gk = workloads.gradient(w, 0, worker=k, device=DEV)
        loco_error_state_init(tmp)
        loco_compensate_quantize(gk, tmp, bits, B, w.beta, False, recv_codes[k * cstride:k * cstride + cb],
                                 recv_scales[k * nb:(k + 1) * nb])
        zero[:] = 0
        ref_codes[k, :cb], ref_scales[k] = oracle.compensate_quantize(host_grad(gk), zero, bits, B, w.beta,
                                                                      threads=threads)
        del gk
    del tmp, zero
    torch.cuda.synchronize()
    assert np.array_equal(recv_codes.cpu().numpy(), ref_codes.reshape(-1)), "a peer's payload differs"
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out)
    want = oracle.dequant_reduce(ref_codes.reshape(-1), ref_scales.reshape(-1), W, n, bits, B, cstride, nb,
                                 threads=threads)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    top = float(np.abs(want).max())
    assert float(np.abs(got - want).max()) <= 1e-6 * top
    bad = int(np.count_nonzero(got != want))
    assert bad == 0, f"{bad} of {n} averaged values differ"
    print(f"[{name}] reduce over W={W}: identical over {n} elements", flush=True)


def test_beyond_two_to_the_32_elements():
    """64-bit indexing: a shard of 2^32 + 2^20 + 333 elements (element indices, and the byte offsets of
    every array, pass 2^31, 2^32 and 2^34).  Blocks on both sides of those boundaries, the ragged last
    block and a few thousand random ones are recomputed by the oracle; the reduce over two payloads is
    checked on the same blocks and must have written every element."""
    n, bits, B, W = (1 << 32) + (1 << 20) + 333, 4, 256, 2
    w = workloads.Workload("beyond_2_32", "gauss", n, torch.bfloat16, bits, B, num_workers=W,
                           segments=(("all", 0, n),))
    nb = loco_num_blocks(n, B)
    cb = loco_code_bytes(n, bits)
    cstride = (cb + 15) // 16 * 16
    rs = np.random.default_rng(32)
    picks = set(rs.integers(0, nb - 1, 3000).tolist())
    for edge in (1 << 29, 1 << 30, 1 << 31, 1 << 32, 1 << 33):      # element index, or byte offset / 1, 2, 4, 8
        for el in (edge, edge // 2, edge // 4, edge * 2):
            b = el // B
            picks.update(x for x in (b - 1, b, b + 1) if 0 <= x < nb - 1)
    picks.update(range(0, 3))
    picks.update(range(nb - 4, nb - 1))
    blocks = np.array(sorted(picks), dtype=np.int64)                # whole blocks; the ragged last one below
    eidx, cidx = element_index(blocks, B), code_index(blocks, B, bits)
    bidx = torch.from_numpy(blocks).to(DEV)
    tail0 = (nb - 1) * B                                            # first element of the last, partial block
    recv_codes = torch.zeros(W * cstride, dtype=torch.uint8, device=DEV)
    recv_scales = torch.zeros(W * nb, dtype=torch.float32, device=DEV)
    err = torch.empty(n, dtype=torch.float32, device=DEV)
    ref_codes = np.zeros((W, cidx.numel()), np.uint8)
    ref_scales = np.zeros((W, blocks.size), np.float32)
    tail_codes, tail_scales = [], []
    for k in range(W):
        g = workloads.gradient(w, 0, worker=k if k else None, device=DEV)
        loco_error_state_init(err)
        e_ref = np.zeros(eidx.numel(), np.float32)
        e_tail = np.zeros(n - tail0, np.float32)
        codes_k, scales_k = recv_codes[k * cstride:k * cstride + cb], recv_scales[k * nb:(k + 1) * nb]
        for step in range(2 if k == 0 else 1):
            loco_compensate_quantize(g, err, bits, B, w.beta, False, codes_k, scales_k)
            ref_codes[k], ref_scales[k] = oracle.compensate_quantize(host_grad(g[eidx]), e_ref, bits, B, w.beta)
            c_tail, s_tail = oracle.compensate_quantize(host_grad(g[tail0:]), e_tail, bits, B, w.beta)
            torch.cuda.synchronize()
            assert np.array_equal(codes_k[cidx].cpu().numpy(), ref_codes[k]), f"worker {k} step {step}: codes"
            assert np.array_equal(scales_k[bidx].cpu().numpy().view(np.uint32), ref_scales[k].view(np.uint32))
            assert np.array_equal(err[eidx].cpu().numpy(), e_ref), f"worker {k} step {step}: state"
            assert np.array_equal(codes_k[tail0 // 2:].cpu().numpy(), c_tail), "codes of the last, partial block"
            assert np.array_equal(scales_k[nb - 1:].cpu().numpy().view(np.uint32), s_tail.view(np.uint32))
            assert np.array_equal(err[tail0:].cpu().numpy(), e_tail)
        tail_codes.append(c_tail)
        tail_scales.append(s_tail)
        del g
    del err
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out)
    torch.cuda.synchronize()
    want = oracle.dequant_reduce(ref_codes.reshape(-1), ref_scales.reshape(-1), W, eidx.numel(), bits, B,
                                 ref_codes.shape[1], ref_scales.shape[1])
    assert np.array_equal(out[eidx].cpu().numpy(), want)
    want_tail = oracle.dequant_reduce(np.concatenate(tail_codes), np.concatenate(tail_scales), W, n - tail0, bits, B,
                                      tail_codes[0].size, 1)
    assert np.array_equal(out[tail0:].cpu().numpy(), want_tail)
    assert bool(torch.isfinite(out).all())
