"""GPU vs CPU oracle for Algorithm 1 exactly as printed (global scale s, 8-bit error state):
loco_compensate_quantize_fixed, loco_dequant_reduce_fixed, loco_error_state8_init.

Bar: gradient codes and state codes bit-exact (both are integers); the fp32 averaged
gradient within 1e-6 relative, and in fact identical.  All calls go through the C ABI.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize_fixed, loco_dequant_reduce_fixed,
                                  loco_error_state8_init, loco_reset_due, workloads)
from paper_2407_04480_amd.binding import LocoError

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def step_both(tag, g_t, e_t, e_host, bits, log2_s, mult, beta, reset=False):
    codes_t = torch.full((loco_code_bytes(g_t.numel(), bits),), 0x5A, dtype=torch.uint8, device=DEV)
    loco_compensate_quantize_fixed(g_t, e_t, bits, log2_s, mult, beta, reset, codes_t)
    c_ref = oracle.fixed_compensate_quantize(workloads.as_numpy_grad(g_t), e_host, bits, log2_s, mult, beta, int(reset))
    torch.cuda.synchronize()
    c_gpu, e_gpu = codes_t.cpu().numpy(), e_t.cpu().numpy()
    assert np.array_equal(c_gpu, c_ref), f"{tag}: {np.count_nonzero(c_gpu != c_ref)} code bytes differ"
    assert np.array_equal(e_gpu, e_host), f"{tag}: {np.count_nonzero(e_gpu != e_host)} state codes differ"
    return c_ref


SHAPES = [1, 7, 8, 9, 15, 16, 17, 511, 512, 513, 1023, 1025, 2047, 2049, 5 * 1024 + 517, 100_003]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("mult", [4, 6])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fixed_cq_small_and_ragged_shapes(bits, mult, dtype):
    log2_s = 19
    qmax = (1 << (bits - 1)) - 1
    rng = torch.Generator(device="cpu").manual_seed(17 * bits + mult)
    for n in SHAPES:
        e_t = torch.full((n,), 77, dtype=torch.int8, device=DEV)
        loco_error_state8_init(e_t)
        assert not e_t.cpu().numpy().any()
        e_host = np.zeros(n, np.int8)
        for step in range(3):
            # a third of the elements clamp, the rest do not
            g = (torch.randn(n, generator=rng) * (0.8 * qmax / 2.0 ** log2_s)).to(dtype)
            step_both(f"n={n} bits={bits} mult={mult} {dtype} step={step}", g.to(DEV), e_t, e_host,
                      bits, log2_s, mult, 0.25)


@pytest.mark.parametrize("mult", [1, 2, 3, 4, 5, 6, 7, 8, 12, 63, 64])
def test_fixed_cq_every_state_value(mult):
    """Every 8-bit state value against many gradients, for power-of-two and other s_e/s:
    exercises the correctly rounded float(e)/s_e for all 256 numerators."""
    bits, log2_s = 4, 17
    n = 256 * 512
    rs = np.random.default_rng(mult)
    e0 = np.repeat(np.arange(-128, 128, dtype=np.int8), 512)
    g = (rs.standard_normal(n) * 4 / 2.0 ** log2_s).astype(np.float32)
    for beta in (0.25, 0.3, 1.0):
        e_t, e_host = torch.from_numpy(e0.copy()).to(DEV), e0.copy()
        step_both(f"all states mult={mult} beta={beta}", torch.from_numpy(g).to(DEV), e_t, e_host,
                  bits, log2_s, mult, beta)


@pytest.mark.parametrize("log2_s", [19, 17, 3, -2, 40])
def test_fixed_cq_scales_beta_reset_and_saturation(log2_s):
    bits, mult, n = 4, 6, 4 * 1024 + 99
    s = 2.0 ** log2_s
    rs = np.random.default_rng(100 + log2_s)
    e_t = torch.zeros(n, dtype=torch.int8, device=DEV)
    e_host = np.zeros(n, np.int8)
    for step, beta in enumerate((0.0, 0.25, 0.5, 1.0, 0.9)):
        g = (rs.standard_normal(n) * rs.choice([0.1, 1, 5, 50, 1e6], n) / s).astype(np.float32)
        g[:8] = 0
        g[8:16] = [1e30, -1e30, 3e38, -3e38, 7.5 / s, -8.5 / s, 0.5 / s, -0.5 / s]
        reset = bool(loco_reset_due(step, 3)) and step > 0
        step_both(f"log2_s={log2_s} step={step}", torch.from_numpy(g).to(DEV), e_t, e_host, bits, log2_s, mult,
                  beta, reset=reset)
        if reset:
            assert not e_host.any()
    assert loco_reset_due(0, 512) and loco_reset_due(1024, 512) and not loco_reset_due(5, 512) and not loco_reset_due(5, 0)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("W", [1, 2, 3, 4, 8, 15, 16, 17, 33, 257, 300])
def test_fixed_dequant_reduce(bits, W):
    """Random codes (every value, including the most negative), padded strides, ragged n.
    W above 16 (4-bit) and above 256 (8-bit) crosses the widening of the packed sums."""
    log2_s = 19
    for n in (5 * 1024 + 333, 7, 1023):
        rs = np.random.default_rng(W * 7 + bits + n)
        cb = oracle.code_bytes(n, bits)
        stride = (cb + 15) // 16 * 16 + 16
        codes = rs.integers(0, 256, W * stride, dtype=np.uint8)
        if W in (17, 300):
            codes[:] = 0x88 if bits == 4 else 0x80      # all workers at the most negative code
        out_t = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
        loco_dequant_reduce_fixed(torch.from_numpy(codes).to(DEV), stride, W, n, bits, log2_s, out_t)
        torch.cuda.synchronize()
        ref = oracle.fixed_dequant_reduce(codes, W, n, bits, log2_s, code_stride_bytes=stride)
        got = out_t.cpu().numpy()
        assert float(np.abs(got - ref).max()) <= 1e-6 * float(np.abs(ref).max())
        assert np.array_equal(got, ref), f"bits={bits} W={W} n={n}: {np.count_nonzero(got != ref)} differ"


@pytest.mark.parametrize("name", workloads.WORKLOAD_NAMES)
def test_fixed_workloads_small(name):
    """The benchmark workloads, shrunk, through the fixed-scale path with the paper's
    constants (s = 2^19, s_e = 4s): every step, then Eq. 8 over W payloads."""
    w = workloads.small(name)
    n, bits, log2_s, mult = w.n, w.bits, 19, 4
    e_t = torch.zeros(n, dtype=torch.int8, device=DEV)
    e_host = np.zeros(n, np.int8)
    for step in range(min(w.steps, 4)):
        g = workloads.gradient(w, step)
        c_own = step_both(f"{w.name} step={step}", g.to(DEV), e_t, e_host, bits, log2_s, mult, w.beta)
    cb = oracle.code_bytes(n, bits)
    stride = (cb + 15) // 16 * 16
    codes = np.zeros(w.num_workers * stride, np.uint8)
    codes[:cb] = c_own
    for k in range(1, w.num_workers):
        gk = workloads.as_numpy_grad(workloads.gradient(w, 0, worker=k))
        codes[k * stride:k * stride + cb] = oracle.fixed_compensate_quantize(gk, np.zeros(n, np.int8), bits, log2_s,
                                                                              mult, w.beta, threads=8)
    out_t = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_dequant_reduce_fixed(torch.from_numpy(codes).to(DEV), stride, w.num_workers, n, bits, log2_s, out_t)
    torch.cuda.synchronize()
    ref = oracle.fixed_dequant_reduce(codes, w.num_workers, n, bits, log2_s, code_stride_bytes=stride)
    assert np.array_equal(out_t.cpu().numpy(), ref)


def test_fixed_full_size_sampled():
    """The 7B shard at full size in the benchmark's launch configuration: elements are
    independent, so the oracle recomputes sampled runs of elements step by step."""
    w = workloads.by_name("llama7b_shard_4bit_b256")
    n, bits, log2_s, mult, W = w.n, 4, 19, 4, 8
    rs = np.random.default_rng(5)
    starts = np.unique(np.concatenate([rs.integers(0, n // 64 - 1, 4000) * 64, [0, n - 64],
                                       (rs.integers(1, n // 1024, 64) * 1024 - 64)]))
    idx = (starts[:, None] + np.arange(64)[None, :]).reshape(-1)
    eidx = torch.from_numpy(idx).to(DEV)
    cidx = torch.from_numpy((starts[:, None] // 2 + np.arange(32)[None, :]).reshape(-1)).to(DEV)
    ns = idx.size
    cb = loco_code_bytes(n, bits)
    stride = (cb + 15) // 16 * 16
    recv = torch.zeros(W * stride, dtype=torch.uint8, device=DEV)
    err = torch.empty(n, dtype=torch.int8, device=DEV)
    loco_error_state8_init(err)
    e_ref = np.zeros(ns, np.int8)
    grads = [workloads.gradient(w, s, device=DEV) * 1e-2 for s in range(2)]   # bring part of it below the clamp
    grads = [g.to(torch.bfloat16) for g in grads]
    ref_codes = np.zeros((W, ns // 2), np.uint8)
    for step in range(4):
        g = grads[step & 1]
        loco_compensate_quantize_fixed(g, err, bits, log2_s, mult, w.beta, False, recv[:cb])
        ref_codes[0] = oracle.fixed_compensate_quantize(workloads.as_numpy_grad(g[eidx]), e_ref, bits, log2_s, mult, w.beta)
        torch.cuda.synchronize()
        assert np.array_equal(recv[:cb][cidx].cpu().numpy(), ref_codes[0]), f"step {step}: codes differ"
        assert np.array_equal(err[eidx].cpu().numpy(), e_ref), f"step {step}: state differs"
    assert 0.001 < float((err != 0).float().mean()) and int(err.abs().max()) <= 128
    tmp = torch.empty(n, dtype=torch.int8, device=DEV)
    for k in range(1, W):
        gk = (workloads.gradient(w, 0, worker=k, device=DEV) * 1e-2).to(torch.bfloat16)
        loco_error_state8_init(tmp)
        loco_compensate_quantize_fixed(gk, tmp, bits, log2_s, mult, w.beta, False, recv[k * stride:k * stride + cb])
        ref_codes[k] = oracle.fixed_compensate_quantize(workloads.as_numpy_grad(gk[eidx]), np.zeros(ns, np.int8),
                                                         bits, log2_s, mult, w.beta)
        del gk
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce_fixed(recv, stride, W, n, bits, log2_s, out)
    torch.cuda.synchronize()
    want = oracle.fixed_dequant_reduce(ref_codes.reshape(-1), W, ns, bits, log2_s, code_stride_bytes=ns // 2)
    assert np.array_equal(out[eidx].cpu().numpy(), want)
    assert bool(torch.isfinite(out).all())


def test_fixed_full_size_every_element(capsys):
    """The 7B shard over the WHOLE array for Algorithm 1 as printed (s = 2^19, s_e = 6s, so the
    state decode takes the corrected-quotient path): two steps, every code byte and every 8-bit
    state value, then Eq. 8 over the W payloads, every element."""
    import os
    w = workloads.by_name("llama7b_shard_4bit_b256")
    n, bits, log2_s, mult, W = w.n, 4, 19, 6, 8
    threads = max(1, min(16, os.cpu_count() or 1))
    cb = loco_code_bytes(n, bits)
    stride = (cb + 15) // 16 * 16
    recv = torch.zeros(W * stride, dtype=torch.uint8, device=DEV)
    ref = np.zeros((W, stride), np.uint8)
    err = torch.empty(n, dtype=torch.int8, device=DEV)
    loco_error_state8_init(err)
    e_ref = np.zeros(n, np.int8)
    for k in range(W):
        for step in range(2 if k == 0 else 1):
            g = (workloads.gradient(w, step, worker=None if k == 0 else k, device=DEV) * 1e-2).to(torch.bfloat16)
            if k:
                loco_error_state8_init(err)
                e_ref[:] = 0
            loco_compensate_quantize_fixed(g, err, bits, log2_s, mult, w.beta, False, recv[k * stride:k * stride + cb])
            ref[k, :cb] = oracle.fixed_compensate_quantize(workloads.as_numpy_grad(g), e_ref, bits, log2_s, mult,
                                                           w.beta, threads=threads)
            torch.cuda.synchronize()
            del g
            assert np.array_equal(recv[k * stride:k * stride + cb].cpu().numpy(), ref[k, :cb]), f"w={k} step={step}: codes"
            assert np.array_equal(err.cpu().numpy(), e_ref), f"w={k} step={step}: state"
            with capsys.disabled():
                print(f"[fixed, whole array] worker {k} step {step}: codes and state identical over {n} elements",
                      flush=True)
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce_fixed(recv, stride, W, n, bits, log2_s, out)
    want = oracle.fixed_dequant_reduce(ref.reshape(-1), W, n, bits, log2_s, code_stride_bytes=stride, threads=threads)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert int(np.count_nonzero(got != want)) == 0


def test_fixed_beyond_two_to_the_32_elements():
    """64-bit indexing of the fixed-scale kernels: 2^32 + 2^20 + 77 elements; runs of 64 elements on
    both sides of 2^29 ... 2^33 (element index or byte offset), the ragged end and random runs are
    recomputed by the oracle, for the compressor (two steps) and for Eq. 8 over two payloads."""
    n, bits, log2_s, mult, W, beta = (1 << 32) + (1 << 20) + 77, 4, 19, 6, 2, 0.25
    rs = np.random.default_rng(33)
    starts = set((rs.integers(0, n // 64 - 2, 3000) * 64).tolist())
    for edge in (1 << 29, 1 << 30, 1 << 31, 1 << 32, 1 << 33):
        for el in (edge, edge // 2, edge * 2):
            starts.update(x for x in (el - 64, el) if 0 <= x <= n - 128)
    starts.update({0, 64})
    starts = np.array(sorted(starts), dtype=np.int64)
    idx = (starts[:, None] + np.arange(64)[None, :]).reshape(-1)
    eidx = torch.from_numpy(idx).to(DEV)
    cidx = torch.from_numpy((starts[:, None] // 2 + np.arange(32)[None, :]).reshape(-1)).to(DEV)
    tail0 = n // 64 * 64 - 64                       # the last whole run and the ragged end behind it
    cb = loco_code_bytes(n, bits)
    stride = (cb + 15) // 16 * 16
    recv = torch.zeros(W * stride, dtype=torch.uint8, device=DEV)
    err = torch.empty(n, dtype=torch.int8, device=DEV)
    wl = workloads.Workload("beyond_2_32", "gauss", n, torch.bfloat16, bits, 256, segments=(("all", 0, n),))
    ref = np.zeros((W, idx.size // 2), np.uint8)
    tails = []
    for k in range(W):
        g = (workloads.gradient(wl, 0, worker=k if k else None, device=DEV) * 1e-2).to(torch.bfloat16)
        loco_error_state8_init(err)
        e_ref, e_tail = np.zeros(idx.size, np.int8), np.zeros(n - tail0, np.int8)
        mine = recv[k * stride:k * stride + cb]
        for step in range(2 if k == 0 else 1):
            loco_compensate_quantize_fixed(g, err, bits, log2_s, mult, beta, False, mine)
            ref[k] = oracle.fixed_compensate_quantize(workloads.as_numpy_grad(g[eidx]), e_ref, bits, log2_s, mult, beta)
            c_tail = oracle.fixed_compensate_quantize(workloads.as_numpy_grad(g[tail0:]), e_tail, bits, log2_s, mult, beta)
            torch.cuda.synchronize()
            assert np.array_equal(mine[cidx].cpu().numpy(), ref[k]), f"worker {k} step {step}: codes"
            assert np.array_equal(err[eidx].cpu().numpy(), e_ref), f"worker {k} step {step}: state"
            assert np.array_equal(mine[tail0 // 2:].cpu().numpy(), c_tail) and np.array_equal(err[tail0:].cpu().numpy(), e_tail)
        tails.append(c_tail)
        del g
    del err
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce_fixed(recv, stride, W, n, bits, log2_s, out)
    torch.cuda.synchronize()
    want = oracle.fixed_dequant_reduce(ref.reshape(-1), W, idx.size, bits, log2_s, code_stride_bytes=idx.size // 2)
    assert np.array_equal(out[eidx].cpu().numpy(), want)
    want_tail = oracle.fixed_dequant_reduce(np.concatenate(tails), W, n - tail0, bits, log2_s,
                                            code_stride_bytes=tails[0].size)
    assert np.array_equal(out[tail0:].cpu().numpy(), want_tail)
    assert bool(torch.isfinite(out).all())


def test_fixed_argument_errors():
    n = 4096
    g = torch.zeros(n, device=DEV)
    e = torch.zeros(n, dtype=torch.int8, device=DEV)
    codes = torch.zeros(n // 2, dtype=torch.uint8, device=DEV)
    for bad in (dict(bits=5), dict(log2_s=65), dict(se_mult=0), dict(se_mult=65)):
        kw = dict(bits=4, log2_s=19, se_mult=4)
        kw.update(bad)
        with pytest.raises(LocoError) as ei:
            loco_compensate_quantize_fixed(g, e, kw["bits"], kw["log2_s"], kw["se_mult"], 0.25, False, codes)
        assert ei.value.status == 2
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize_fixed(g, e, 4, 19, 4, 1.25, False, codes)
    assert ei.value.status == 1
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize_fixed(g[1:], e[1:], 4, 19, 4, 0.25, False, codes)
    assert ei.value.status == 3
    out = torch.zeros(n, device=DEV)
    with pytest.raises(LocoError) as ei:
        loco_dequant_reduce_fixed(codes, 8, 2, 64, 4, 19, out)      # stride shorter than a payload
    assert ei.value.status == 1
    torch.cuda.synchronize()


# ---- global scale with the compensation error kept in fp32 (ablation row without error compression) ----
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fixed_f32state_small_and_ragged_shapes(bits, dtype):
    from paper_2407_04480_amd import loco_compensate_quantize_fixed_f32state, loco_error_state_init
    rng = torch.Generator(device="cpu").manual_seed(500 + bits + (dtype == torch.bfloat16))
    qmax = (1 << (bits - 1)) - 1
    for n in SHAPES + [6 * 2048 + 1031]:
        for log2_s, beta in ((19, 0.25), (17, 1.0), (3, 0.3)):
            e_t = torch.full((n,), 3.0, dtype=torch.float32, device=DEV)
            loco_error_state_init(e_t)
            e_host = np.zeros(n, np.float32)
            for step in range(3):
                g = (torch.randn(n, generator=rng) * (0.6 * qmax / 2.0 ** log2_s)).to(dtype)   # some clamp
                codes_t = torch.full((loco_code_bytes(n, bits),), 0x5A, dtype=torch.uint8, device=DEV)
                reset = step == 1 and beta == 0.3
                loco_compensate_quantize_fixed_f32state(g.to(DEV), e_t, bits, log2_s, beta, reset, codes_t)
                c_ref = oracle.fixed_compensate_quantize_f32state(workloads.as_numpy_grad(g), e_host, bits, log2_s, beta,
                                                                  int(reset))
                torch.cuda.synchronize()
                tag = f"n={n} bits={bits} {dtype} s=2^{log2_s} beta={beta} step={step}"
                assert np.array_equal(codes_t.cpu().numpy(), c_ref), f"{tag}: codes differ"
                e_gpu = e_t.cpu().numpy()
                assert np.array_equal(e_gpu, e_host), f"{tag}: {np.count_nonzero(e_gpu != e_host)} state values differ"


def test_fixed_f32state_full_size_every_element(capsys):
    """The 7B shard, whole array, two steps; then Eq. 8 over payloads of this form."""
    from paper_2407_04480_amd import loco_compensate_quantize_fixed_f32state, loco_error_state_init
    w = workloads.by_name("llama7b_shard_4bit_b256")
    n, bits, log2_s, W = w.n, 4, 19, 3
    cb = loco_code_bytes(n, bits)
    stride = (cb + 15) // 16 * 16
    recv = torch.zeros(W * stride, dtype=torch.uint8, device=DEV)
    ref = np.zeros((W, stride), np.uint8)
    err = torch.empty(n, dtype=torch.float32, device=DEV)
    e_ref = np.zeros(n, np.float32)
    for k in range(W):
        loco_error_state_init(err)
        e_ref[:] = 0
        for step in range(2 if k == 0 else 1):
            g = (workloads.gradient(w, step, worker=None if k == 0 else k, device=DEV) * 1e-2).to(torch.bfloat16)
            loco_compensate_quantize_fixed_f32state(g, err, bits, log2_s, w.beta, False, recv[k * stride:k * stride + cb])
            ref[k, :cb] = oracle.fixed_compensate_quantize_f32state(workloads.as_numpy_grad(g), e_ref, bits, log2_s, w.beta)
            torch.cuda.synchronize()
            del g
            assert np.array_equal(recv[k * stride:k * stride + cb].cpu().numpy(), ref[k, :cb]), f"w={k} step={step}: codes"
            e_gpu = err.cpu().numpy()
            assert np.array_equal(e_gpu, e_ref), f"w={k} step={step}: {np.count_nonzero(e_gpu != e_ref)} state values"
            with capsys.disabled():
                print(f"[fixed, fp32 state, whole array] worker {k} step {step}: identical over {n} elements", flush=True)
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce_fixed(recv, stride, W, n, bits, log2_s, out)
    want = oracle.fixed_dequant_reduce(ref.reshape(-1), W, n, bits, log2_s, code_stride_bytes=stride, threads=16)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)


def test_fixed_f32state_argument_errors():
    from paper_2407_04480_amd import loco_compensate_quantize_fixed_f32state
    n = 4096
    g = torch.zeros(n, device=DEV)
    e = torch.zeros(n, device=DEV)
    codes = torch.zeros(n // 2, dtype=torch.uint8, device=DEV)
    for kw, status in ((dict(bits=5), 2), (dict(log2_s=65), 2), (dict(beta=1.5), 1), (dict(beta=float("nan")), 1)):
        a = dict(bits=4, log2_s=19, beta=0.25)
        a.update(kw)
        with pytest.raises(LocoError) as ei:
            loco_compensate_quantize_fixed_f32state(g, e, a["bits"], a["log2_s"], a["beta"], False, codes)
        assert ei.value.status == status
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize_fixed_f32state(g[1:], e[1:], 4, 19, 0.25, False, codes)
    assert ei.value.status == 3
    torch.cuda.synchronize()
