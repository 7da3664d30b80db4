"""The seeded input generator (paper_2407_04480_amd/workloads.py): every element is a pure
function of (seed, step, worker, tensor, index), so the bytes do not depend on the chunking or
on the device; the recipes have the distributions the workloads state."""
import numpy as np
import pytest
import torch

from paper_2407_04480_amd import workloads

SMALL = list(workloads.WORKLOAD_NAMES)


def bits_of(t: torch.Tensor) -> np.ndarray:
    return workloads.as_numpy_grad(t).view(np.uint16 if t.dtype == torch.bfloat16 else np.uint32)


@pytest.mark.parametrize("name", SMALL)
def test_same_bytes_for_any_chunking(name):
    w = workloads.small(name)
    a = bits_of(workloads.gradient(w, 2, worker=1))
    for chunk in (1 << 30, 4099, 1 << 12):
        assert np.array_equal(a, bits_of(workloads.gradient(w, 2, worker=1, chunk=chunk)))


def test_keys_separate_steps_workers_and_tensors():
    w = workloads.small("llama7b_shard_4bit_b256")
    base = bits_of(workloads.gradient(w, 0))
    for other in (workloads.gradient(w, 1), workloads.gradient(w, 0, worker=0), workloads.gradient(w, 0, worker=1)):
        same = np.count_nonzero(bits_of(other) == base) / base.size
        assert same < 0.02                       # bf16 has few values: chance agreement only
    assert np.array_equal(base, bits_of(workloads.gradient(w, 0)))
    keys = {workloads.stream_key(workloads.BASE_SEED, s, k, t) for s in range(4) for k in (None, 0, 1, 2) for t in range(5)}
    assert len(keys) == 4 * 4 * 5
    # the same index in two tensors of one gradient draws different numbers
    (_, s0, l0), (_, s1, l1) = w.segments[1], w.segments[2]
    m = min(l0, l1, 4096)
    f = workloads._tensor_factors(w, -5.0, -2.0)
    g = workloads.gradient(w, 0).double()
    assert not torch.allclose(g[s0:s0 + m] / f[1], g[s1:s1 + m] / f[2], rtol=0.02)


def test_normal_recipe_is_normal():
    w = workloads.gauss_1m()
    x = workloads.gradient(w, 0).double() / 1e-3
    n = x.numel()
    assert abs(float(x.mean())) < 4 / np.sqrt(n)
    assert abs(float(x.var()) - 1) < 0.01
    assert abs(float((x ** 4).mean()) - 3) < 0.05
    for z, p in ((1.0, 0.31731), (1.959964, 0.05), (3.290527, 0.001)):
        frac = float((x.abs() > z).double().mean())
        assert abs(frac - p) < 5 * np.sqrt(p / n) + 1e-5, (z, frac)
    assert 4.5 < float(x.abs().max()) < 7


def test_student_t_recipe_has_three_degrees_of_freedom():
    n = 1 << 21
    w = workloads.Workload("t3", "student_t", n, torch.float32, 4, 256, segments=(("all", 0, n),))
    fac = workloads._tensor_factors(w, -5.0, -2.0)[0]
    assert 1e-5 <= fac <= 1e-2
    x = workloads.gradient(w, 0).double() / fac
    for t, p in ((0.7648923, 0.5), (2.353363, 0.1), (3.182446, 0.05), (5.840909, 0.01), (12.92398, 0.001)):
        frac = float((x.abs() > t).double().mean())      # two-sided tail probabilities of t(3)
        assert abs(frac - p) < 5 * np.sqrt(p / n) + 2e-5, (t, frac)
    assert float(x.abs().max()) > 50                      # heavy tail: far beyond any normal sample


def test_outlier_and_moe_recipes():
    w = workloads.small("dense70b_shard_4bit_b256")
    x = workloads.gradient(w, 0).double()
    big = float((x.abs() > 0.01).double().mean())         # 10 sigma of the bulk, 0.1 sigma of an outlier
    assert abs(big - 1e-3 * 0.92) < 2e-4                  # P(|Z| > 0.1) = 0.92 of the 0.1 % outliers
    assert abs(float(x[x.abs() < 0.006].std()) - 1e-3) < 2e-5
    m = workloads.small("mixtral_moe_shard_4bit_b128")
    g = workloads.gradient(m, 3).double()
    fac = workloads._tensor_factors(m, -6.0, -3.0)
    for e, (_, start, length) in enumerate(m.segments):
        part = g[start:start + length]
        if e in workloads.ZERO_EXPERTS:
            assert not bool(part.any())
        else:
            assert 1e-6 <= fac[e] <= 1e-3 and abs(float(part.std()) / fac[e] - 1) < 0.02


@pytest.mark.gpu
@pytest.mark.parametrize("name", SMALL)
def test_cpu_and_gpu_generate_the_same_bytes(name):
    w = workloads.small(name)
    for step, worker in ((0, None), (1, None), (0, 2)):
        cpu = bits_of(workloads.gradient(w, step, worker=worker, device="cpu"))
        gpu = bits_of(workloads.gradient(w, step, worker=worker, device="cuda:0", chunk=1 << 18))
        assert np.array_equal(cpu, gpu), f"{name} step {step} worker {worker}: {np.count_nonzero(cpu != gpu)} differ"


@pytest.mark.gpu
def test_full_size_generation_matches_cpu_on_samples():
    """The headline workload generated on the GPU at full size: slices recomputed on the CPU."""
    w = workloads.by_name("llama7b_shard_4bit_b256")
    g = workloads.gradient(w, 0, device="cuda:0")
    for (_, start, length) in (w.segments[0], w.segments[5], w.segments[-1]):
        take = min(length, 50_000)
        # same tensor index and in-tensor positions: regenerate the piece on the CPU through the key
        t = [s[1] for s in w.segments].index(start)
        key = workloads.stream_key(workloads.BASE_SEED, 0, None, t)
        x = workloads.random_bits(key, 0, take, "cpu")
        fac = workloads._tensor_factors(w, -5.0, -2.0)[t]
        v = (workloads._symmetric_from_bits(workloads._hi32(x), "student_t3") * fac).to(torch.float32).to(w.grad_dtype)
        assert np.array_equal(bits_of(v), bits_of(g[start:start + take])), f"tensor {t}"
