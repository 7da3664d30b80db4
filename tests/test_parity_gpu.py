"""GPU library vs CPU oracle, element by element, on the same seeded inputs.

Bar: packed codes and per-block steps bit-exact; fp32 error state and averaged
gradient within 1e-6 relative (of the tensor's largest magnitude).  Because both
sides perform the same binary32 operations in the same order, the tests also
require the fp32 outputs to be bit-identical and say how many are not if that fails.
Every call goes through the C ABI (ctypes binding).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize, loco_dequant_reduce,
                                  loco_error_state_init, loco_num_blocks, workloads)
from paper_2407_04480_amd.binding import LocoError

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
REL_TOL = 1e-6


def bits_equal_f32(a: np.ndarray, b: np.ndarray) -> int:
    return int(np.count_nonzero(a.view(np.uint32) != b.view(np.uint32)))


def assert_f32_close(name, got: np.ndarray, want: np.ndarray):
    top = float(np.abs(want).max()) if want.size else 0.0
    err = float(np.abs(got.astype(np.float64) - want.astype(np.float64)).max()) if want.size else 0.0
    assert err <= REL_TOL * top, f"{name}: max abs err {err} > 1e-6 * {top}"
    # same operations in the same order: bit-identical, up to the sign of zero
    diff = np.count_nonzero(got != want)
    assert diff == 0, f"{name}: {diff} of {want.size} values differ although within tolerance"


def gpu_cq(g: torch.Tensor, e: torch.Tensor, bits, B, beta, reset=False):
    n = g.numel()
    codes = torch.full((loco_code_bytes(n, bits),), 0xAA, dtype=torch.uint8, device=g.device)
    scales = torch.full((loco_num_blocks(n, B),), -1.0, dtype=torch.float32, device=g.device)
    loco_compensate_quantize(g, e, bits, B, beta, reset, codes, scales)
    return codes, scales


def compare_cq_step(tag, g_t, e_t, e_host, bits, B, beta, reset=False):
    """One step on both sides from the same state; returns the payload (host)."""
    g_host = workloads.as_numpy_grad(g_t)
    codes_t, scales_t = gpu_cq(g_t, e_t, bits, B, beta, reset)
    torch.cuda.synchronize()
    c_ref, s_ref = oracle.compensate_quantize(g_host, e_host, bits, B, beta, int(reset))
    c_gpu, s_gpu, e_gpu = codes_t.cpu().numpy(), scales_t.cpu().numpy(), e_t.cpu().numpy()
    assert np.array_equal(c_gpu, c_ref), f"{tag}: {np.count_nonzero(c_gpu != c_ref)} code bytes differ"
    assert bits_equal_f32(s_gpu, s_ref) == 0, f"{tag}: {bits_equal_f32(s_gpu, s_ref)} block steps differ"
    assert_f32_close(tag + " state", e_gpu, e_host)
    return c_ref, s_ref


SHAPES = [1, 7, 8, 9, 31, 32, 33, 63, 64, 65, 255, 256, 257, 511, 513, 2047, 2048, 2049, 4097,
          6 * 2048 + 1031, 100_003]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("B", [32, 64, 128, 256, 512])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_cq_small_and_ragged_shapes(bits, B, dtype):
    rng = torch.Generator(device="cpu").manual_seed(1000 * bits + B + (dtype == torch.bfloat16))
    for n in SHAPES:
        e_t = torch.empty(n, dtype=torch.float32, device=DEV).fill_(3.0)
        loco_error_state_init(e_t)
        e_host = np.zeros(n, np.float32)
        assert not e_t.cpu().numpy().any()
        for step in range(3):
            g = (torch.randn(n, generator=rng) * 1e-3).to(dtype)
            compare_cq_step(f"n={n} bits={bits} B={B} {dtype} step={step}", g.to(DEV), e_t, e_host,
                            bits, B, 0.25)


@pytest.mark.parametrize("beta", [0.0, 0.25, 0.3, 1.0])
def test_cq_beta_values_and_reset(beta):
    n, bits, B = 3 * 2048 + 77, 4, 256
    rng = torch.Generator(device="cpu").manual_seed(77)
    e_t = torch.zeros(n, dtype=torch.float32, device=DEV)
    e_host = np.zeros(n, np.float32)
    for step in range(4):
        g = torch.randn(n, generator=rng) * 1e-3
        compare_cq_step(f"beta={beta} step={step}", g.to(DEV), e_t, e_host, bits, B, beta,
                        reset=(step == 2))
        if step == 2:
            assert not e_t.cpu().numpy().any()


def test_cq_special_values():
    """Zero blocks, a single non-zero, +-max ties, exact half-way ties, subnormal steps,
    and magnitudes spread over many binades."""
    bits_blocks = [(4, 64), (8, 64), (4, 256), (8, 32)]
    for bits, B in bits_blocks:
        qmax = (1 << (bits - 1)) - 1
        n = 40 * B + 5
        rs = np.random.default_rng(5 + bits + B)
        g = (rs.standard_normal(n) * np.exp2(rs.integers(-30, 4, n))).astype(np.float32)
        g[0:B] = 0                                            # all-zero block
        g[B:2 * B] = 0
        g[B + 3] = 1.25e-3                                    # single non-zero
        g[2 * B:3 * B] = rs.choice([-1.0, 1.0], B) * 2.0 ** -9    # every element at +-max
        m = rs.integers(-2 * qmax, 2 * qmax + 1, B)           # half-integers of the step: ties
        m[0] = 2 * qmax
        g[3 * B:4 * B] = (m * 2.0 ** -14).astype(np.float32)
        g[4 * B:5 * B] = (rs.uniform(-1, 1, B) * 2.0 ** -127).astype(np.float32)   # subnormal step
        g[5 * B:6 * B] = 0
        g[5 * B + 1] = np.float32(qmax) * np.finfo(np.float32).tiny               # smallest live step
        g[5 * B + 2] = -np.float32(3) * np.finfo(np.float32).tiny
        g[6 * B:7 * B] = (rs.uniform(-1, 1, B) * 1e30).astype(np.float32)         # huge
        e_t = torch.zeros(n, dtype=torch.float32, device=DEV)
        e_host = np.zeros(n, np.float32)
        for step in range(3):
            compare_cq_step(f"special bits={bits} B={B} step={step}", torch.from_numpy(g).to(DEV),
                            e_t, e_host, bits, B, 0.5)


def make_payloads(w: workloads.Workload, device=DEV):
    """W peers' payloads in one receive buffer: each is compensate-quantize of an
    independently seeded gradient from a zero state (made by the oracle)."""
    n, bits, B, W = w.n, w.bits, w.block_size, w.num_workers
    cb, nb = oracle.code_bytes(n, bits), oracle.num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    codes = np.zeros(W * cstride, np.uint8)
    scales = np.zeros(W * nb, np.float32)
    for k in range(W):
        g = workloads.as_numpy_grad(workloads.gradient(w, 0, worker=k))
        c, s = oracle.compensate_quantize(g, np.zeros(n, np.float32), bits, B, w.beta, threads=8)
        codes[k * cstride:k * cstride + cb] = c
        scales[k * nb:(k + 1) * nb] = s
    return codes, cstride, scales, nb


@pytest.mark.parametrize("name", workloads.WORKLOAD_NAMES)
def test_workloads_small(name):
    """The five benchmark workloads, shrunk: every step of compensate-quantize, then
    dequant-reduce of W payloads."""
    w = workloads.small(name)
    e_t = torch.zeros(w.n, dtype=torch.float32, device=DEV)
    e_host = np.zeros(w.n, np.float32)
    sum_d = np.zeros(w.n)
    sum_g = np.zeros(w.n)
    for step in range(w.steps):
        g = workloads.gradient(w, step % 2 if w.recipe == "moe" else step)
        c, s = compare_cq_step(f"{w.name} step={step}", g.to(DEV), e_t, e_host, w.bits, w.block_size, w.beta)
        sum_d += oracle.dequant_reduce(c, s, 1, w.n, w.bits, w.block_size)
        sum_g += g.float().numpy()
    # Lemma 1 telescoped (uncompressed state): sum d = sum g - e_K / beta, on the GPU's state
    gmax = float(np.abs(sum_g).max()) + 1e-30
    assert np.abs(sum_d - (sum_g - e_t.cpu().numpy() / w.beta)).max() <= w.steps * 2.0 ** -18 * gmax

    codes, cstride, scales, sstride = make_payloads(w)
    out_t = torch.full((w.n,), 7.0, dtype=torch.float32, device=DEV)
    loco_dequant_reduce(torch.from_numpy(codes).to(DEV), cstride, torch.from_numpy(scales).to(DEV), sstride,
                        w.num_workers, w.n, w.bits, w.block_size, out_t)
    torch.cuda.synchronize()
    ref = oracle.dequant_reduce(codes, scales, w.num_workers, w.n, w.bits, w.block_size, cstride, sstride)
    assert_f32_close(f"{w.name} reduce W={w.num_workers}", out_t.cpu().numpy(), ref)


@pytest.mark.parametrize("bits,B", [(4, 32), (4, 256), (8, 64), (8, 512)])
@pytest.mark.parametrize("W", [1, 2, 3, 5, 8, 16, 17])
def test_dequant_reduce_worker_counts(bits, B, W):
    n = 5 * 2048 + 333
    w = workloads.Workload("t", "gauss", n, torch.float32, bits, B, num_workers=W,
                           segments=(("all", 0, n),))
    codes, cstride, scales, sstride = make_payloads(w)
    pad = 5  # scale stride larger than needed
    scales2 = np.zeros(W * (sstride + pad), np.float32)
    for k in range(W):
        scales2[k * (sstride + pad):k * (sstride + pad) + sstride] = scales[k * sstride:(k + 1) * sstride]
    out_t = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_dequant_reduce(torch.from_numpy(codes).to(DEV), cstride, torch.from_numpy(scales2).to(DEV),
                        sstride + pad, W, n, bits, B, out_t)
    torch.cuda.synchronize()
    ref = oracle.dequant_reduce(codes, scales2, W, n, bits, B, cstride, sstride + pad)
    assert_f32_close(f"reduce bits={bits} B={B} W={W}", out_t.cpu().numpy(), ref)


@pytest.mark.parametrize("bits,B", [(4, 256), (4, 64), (8, 64), (4, 512), (8, 32)])
def test_dequant_reduce_arbitrary_payloads(bits, B):
    """Payloads that compensate-quantize would never emit: every code value including
    -2^(p-1), steps that are huge (16*D overflows), tiny, zero or negative."""
    n, W = 7 * 2048 + 129, 6
    rs = np.random.default_rng(99 + bits + B)
    cb, nb = oracle.code_bytes(n, bits), oracle.num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    codes = rs.integers(0, 256, W * cstride, dtype=np.uint8)
    pool = np.array([0.0, 1e-4, -3e-5, 2.0 ** -126, 2.0 ** -140, 2.0 ** 119, 2.0 ** 120, 2.0 ** 121, 2.0 ** 124,
                     3.0e38 / 127, -(2.0 ** 122), 1.0, 7.25e-3], dtype=np.float32)
    scales = pool[rs.integers(0, pool.size, W * nb)]
    scales[rs.random(W * nb) < 0.7] = np.float32(1e-4)      # most blocks ordinary
    out_t = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_dequant_reduce(torch.from_numpy(codes).to(DEV), cstride, torch.from_numpy(scales).to(DEV), nb,
                        W, n, bits, B, out_t)
    torch.cuda.synchronize()
    with np.errstate(over="ignore", invalid="ignore"):
        ref = oracle.dequant_reduce(codes, scales, W, n, bits, B, cstride, nb)
    got = out_t.cpu().numpy()
    fin = np.isfinite(ref)
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isinf(got), np.isinf(ref))
    assert np.array_equal(got[fin], ref[fin]), f"{np.count_nonzero(got[fin] != ref[fin])} values differ"
    assert fin.mean() > 0.3


@pytest.mark.parametrize("n", [1, 7, 9, 255, 2047, 2049, 100_003])
def test_dequant_reduce_ragged(n):
    for bits, B in ((4, 64), (8, 128)):
        w = workloads.Workload("t", "gauss", n, torch.float32, bits, B, num_workers=3,
                               segments=(("all", 0, n),))
        codes, cstride, scales, sstride = make_payloads(w)
        out_t = torch.empty(n, dtype=torch.float32, device=DEV)
        loco_dequant_reduce(torch.from_numpy(codes).to(DEV), cstride, torch.from_numpy(scales).to(DEV),
                            sstride, 3, n, bits, B, out_t)
        torch.cuda.synchronize()
        ref = oracle.dequant_reduce(codes, scales, 3, n, bits, B, cstride, sstride)
        assert_f32_close(f"reduce ragged n={n} bits={bits}", out_t.cpu().numpy(), ref)


def test_w1_reduce_returns_senders_decode():
    """Alg. 1: the receiver decodes with the sender's own step, so N = 1 gives back d."""
    n, bits, B = 9 * 2048 + 5, 4, 256
    g = (torch.randn(n, generator=torch.Generator().manual_seed(3)) * 1e-3).to(DEV)
    e_t = torch.zeros(n, dtype=torch.float32, device=DEV)
    codes, scales = gpu_cq(g, e_t, bits, B, 1.0)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    loco_dequant_reduce(codes, 0, scales, 0, 1, n, bits, B, out)
    torch.cuda.synchronize()
    # beta = 1: the state is h - d, so d + state == g exactly wherever h - d was exact
    back = (out + e_t).cpu().numpy()
    assert np.count_nonzero(back != g.cpu().numpy()) <= 1e-3 * n
    assert np.abs(back - g.cpu().numpy()).max() <= 2.0 ** -23 * float(g.abs().max())


def test_pointer_and_argument_errors_on_gpu():
    n = 4096
    g = torch.zeros(n, device=DEV)
    e = torch.zeros(n, device=DEV)
    codes = torch.zeros(n // 2, dtype=torch.uint8, device=DEV)
    scales = torch.zeros(n // 256, device=DEV)
    with pytest.raises(LocoError) as ei:      # misaligned view
        loco_compensate_quantize(g[1:], e[1:], 4, 256, 0.25, False, codes, scales)
    assert ei.value.status == 3
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize(g, e, 5, 256, 0.25, False, codes, scales)
    assert ei.value.status == 2
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize(g, e, 4, 256, -0.1, False, codes, scales)
    assert ei.value.status == 1
    with pytest.raises(ValueError):
        loco_compensate_quantize(g, e, 4, 256, 0.25, False, codes[:100], scales)
    # a host pointer is refused by the library itself (ctypes level, no kernel is launched)
    import ctypes
    from paper_2407_04480_amd.binding import load_library
    lib = load_library()
    host = np.zeros(n, np.float32)
    st = lib.loco_error_state_init(ctypes.c_void_p(host.ctypes.data), n, None)
    assert st == 5
    torch.cuda.synchronize()


@pytest.mark.parametrize("nbytes", [16, 1008, 1024, 4096 + 16, 3 * 65536 + 48, (1 << 24) + 16])
def test_stream_measurement_aids(nbytes):
    """The plain copy / read / fill kernels behind bench.py's ceilings do what they say."""
    from paper_2407_04480_amd import loco_stream_copy, loco_stream_fill, loco_stream_read, loco_stream_sum2
    rng = torch.Generator(device="cpu").manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes,), generator=rng, dtype=torch.uint8).to(DEV)
    dst = torch.full((nbytes + 16,), 0x5A, dtype=torch.uint8, device=DEV)
    loco_stream_copy(dst[:nbytes], src)
    torch.cuda.synchronize()
    assert torch.equal(dst[:nbytes], src) and int(dst[nbytes:].min()) == 0x5A     # nothing past the end
    sink = torch.full((16,), 0x33, dtype=torch.uint8, device=DEV)
    before = src.clone()
    loco_stream_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, before)
    other = torch.randint(0, 256, (nbytes,), generator=rng, dtype=torch.uint8).to(DEV)
    loco_stream_sum2(dst[:nbytes], src, other)
    torch.cuda.synchronize()
    want = (src.view(torch.int32) + other.view(torch.int32)).view(torch.uint8)     # wraps, like the kernel
    assert torch.equal(dst[:nbytes], want) and int(dst[nbytes:].min()) == 0x5A
    loco_stream_fill(dst[:nbytes])
    torch.cuda.synchronize()
    assert int(dst[:nbytes].max()) == 0 and int(dst[nbytes:].min()) == 0x5A


@pytest.mark.parametrize("n", [1, 3, 4, 1023, 1024, 1025, 4099, 1 << 20])
def test_state_init_sizes(n):
    """Both state initialisers write exactly n zeros (Eq. 5: e~_0 = 0) and nothing beyond."""
    from paper_2407_04480_amd import loco_error_state8_init
    pad = 16
    e = torch.full((n + pad,), 7.0, dtype=torch.float32, device=DEV)
    loco_error_state_init(e[:n])
    e8 = torch.full((n + pad,), 7, dtype=torch.int8, device=DEV)
    loco_error_state8_init(e8[:n])
    torch.cuda.synchronize()
    assert not e[:n].any() and bool((e[n:] == 7.0).all())
    assert not e8[:n].any() and bool((e8[n:] == 7).all())


def test_resume_from_saved_state():
    """The error state (and the step index, for the reset schedule) is all that persists between
    steps: a run that saves the state to the host after step 3, frees it, reloads it into a new
    allocation and carries on gives the bytes of the uninterrupted run."""
    n, bits, B, beta, K = 9 * 2048 + 517, 4, 128, 0.25, 7
    rng = torch.Generator(device="cpu").manual_seed(4242)
    grads = [(torch.randn(n, generator=rng) * 1e-3).to(torch.bfloat16).to(DEV) for _ in range(K)]

    def run(interrupt_after=None):
        e = torch.empty(n, dtype=torch.float32, device=DEV)
        loco_error_state_init(e)
        trace = []
        for k in range(K):
            codes, scales = gpu_cq(grads[k], e, bits, B, beta, reset=(k == 5))
            trace.append((codes.cpu(), scales.cpu()))
            if interrupt_after == k:
                saved = e.cpu().clone()
                del e
                torch.cuda.empty_cache()
                e = saved.to(DEV)
        torch.cuda.synchronize()
        return trace, e.cpu()

    straight, e_straight = run()
    resumed, e_resumed = run(interrupt_after=3)
    for k in range(K):
        assert torch.equal(straight[k][0], resumed[k][0]), f"step {k}: codes differ after the resume"
        assert torch.equal(straight[k][1].view(torch.int32), resumed[k][1].view(torch.int32)), f"step {k}: steps"
    assert torch.equal(e_straight.view(torch.int32), e_resumed.view(torch.int32))


@pytest.mark.parametrize("bits,B", [(4, 32), (4, 256), (8, 64), (8, 512)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_cq_with_other_residency_gives_the_same_bytes(bits, B, dtype):
    """The measurement variant with 6 or 8 resident wavefronts per SIMD: same codes, steps and state as the
    oracle; values the library does not build are refused."""
    from paper_2407_04480_amd import loco_compensate_quantize_resident
    rng = torch.Generator(device="cpu").manual_seed(4100 + B + bits)
    for waves in (4, 6, 8):
        for n in (1, 513, 6 * 2048 + 1031, 100_003):
            e_t = torch.zeros(n, dtype=torch.float32, device=DEV)
            e_host = np.zeros(n, np.float32)
            for step in range(2):
                g = (torch.randn(n, generator=rng) * 1e-3).to(dtype)
                codes = torch.full((loco_code_bytes(n, bits),), 0xAA, dtype=torch.uint8, device=DEV)
                scales = torch.full((loco_num_blocks(n, B),), -1.0, dtype=torch.float32, device=DEV)
                loco_compensate_quantize_resident(g.to(DEV), e_t, bits, B, 0.25, False, codes, scales, waves)
                c_ref, s_ref = oracle.compensate_quantize(workloads.as_numpy_grad(g), e_host, bits, B, 0.25)
                torch.cuda.synchronize()
                assert np.array_equal(codes.cpu().numpy(), c_ref), f"waves={waves} n={n} step={step}: codes"
                assert bits_equal_f32(scales.cpu().numpy(), s_ref) == 0 and np.array_equal(e_t.cpu().numpy(), e_host)
    g = torch.zeros(512, device=DEV)
    with pytest.raises(LocoError) as ei:
        loco_compensate_quantize_resident(g, torch.zeros_like(g), 4, 256, 0.25, False,
                                          torch.zeros(256, dtype=torch.uint8, device=DEV), torch.zeros(2, device=DEV), 5)
    assert ei.value.status == 2


@pytest.mark.parametrize("B", [32, 64, 128, 256, 512])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_cq_staged_code_stores_give_the_same_bytes(B, dtype):
    """The measurement variant that stages 4-bit codes through LDS: same codes, steps and state as the oracle."""
    from paper_2407_04480_amd import loco_compensate_quantize_staged_codes
    rng = torch.Generator(device="cpu").manual_seed(4000 + B)
    for n in (1, 511, 512, 513, 4096, 6 * 2048 + 1031, 100_003):
        e_t = torch.zeros(n, dtype=torch.float32, device=DEV)
        e_host = np.zeros(n, np.float32)
        for step in range(2):
            g = (torch.randn(n, generator=rng) * 1e-3).to(dtype)
            codes = torch.full((loco_code_bytes(n, 4),), 0xAA, dtype=torch.uint8, device=DEV)
            scales = torch.full((loco_num_blocks(n, B),), -1.0, dtype=torch.float32, device=DEV)
            loco_compensate_quantize_staged_codes(g.to(DEV), e_t, 4, B, 0.25, False, codes, scales)
            c_ref, s_ref = oracle.compensate_quantize(workloads.as_numpy_grad(g), e_host, 4, B, 0.25)
            torch.cuda.synchronize()
            assert np.array_equal(codes.cpu().numpy(), c_ref), f"n={n} B={B} step={step}: codes"
            assert bits_equal_f32(scales.cpu().numpy(), s_ref) == 0 and np.array_equal(e_t.cpu().numpy(), e_host)
