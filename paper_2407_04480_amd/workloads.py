"""Seeded synthetic gradients with the shapes of the benchmark workloads.

This module only makes inputs.  It holds none of the method's arithmetic (no
compensation, no quantisation, no averaging) and imports neither the GPU
binding nor the CPU oracle, so both sides can be fed the very same bytes.

The method (LoCo, arXiv 2407.04480) is measured by its authors inside LLM
training runs (Tables 7 and 10: LLAMA2 7B-70B, Mixtral 8x7B).  Those runs,
their data and their checkpoints are not available here; the gradients below
take only the shapes of such models and stand in for them:

  gauss_1m            2^20 fp32 values ~ N(0, (1e-3)^2)
  llama7b_shard       first 1/8 of the flat gradient of a Llama-style 7B model
                      (embedding, 32 x [4 attention 4096x4096, 3 MLP 4096x11008,
                      2 norms], final norm, head); bf16; per tensor Student-t
                      (3 degrees of freedom) times 10^U, U ~ Uniform[-5, -2]
  mixtral_moe_shard   8 experts x 3 matrices 4096x14336, bf16; experts 1, 4, 6 all
                      zero (not routed to), the others N(0, sigma_e^2) with
                      sigma_e = 10^U, U ~ Uniform[-6, -3]
  dense70b_shard      2.2e9 contiguous bf16 values ~ N(0, (1e-3)^2), each
                      multiplied by 100 with probability 1e-3

Random numbers come from torch generators seeded with BASE_SEED + step (own
gradient) or BASE_SEED + 1000*(worker+1) + step (a peer's gradient); per-tensor
factors come from a CPU generator so they do not depend on the device.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import torch

BASE_SEED = 20240704
# The paper gives no value for the moving-average coefficient of Eq. 5 (only
# 0 <= beta <= 1); benchmarks here use a dyadic value so that beta and 1-beta are
# exact.  Throughput does not depend on it.
DEFAULT_BETA = 0.25

Segment = Tuple[str, int, int]  # (tensor name, first element, length) inside the shard


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    recipe: str                      # 'gauss' | 'student_t' | 'moe' | 'outlier'
    n: int
    grad_dtype: torch.dtype
    bits: int
    block_size: int
    beta: float = DEFAULT_BETA
    num_workers: int = 1
    steps: int = 3
    segments: Tuple[Segment, ...] = ()
    note: str = ""

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def llama_segments(hidden: int, ffn: int, vocab: int, layers: int, shard: int = 8) -> Tuple[int, List[Segment]]:
    """Flat parameter order of a Llama-style model, cut to the first 1/shard."""
    tensors: List[Tuple[str, int]] = [("embed", vocab * hidden)]
    for l in range(layers):
        for nm in ("wq", "wk", "wv", "wo"):
            tensors.append((f"l{l}.{nm}", hidden * hidden))
        for nm in ("w_gate", "w_up", "w_down"):
            tensors.append((f"l{l}.{nm}", hidden * ffn))
        for nm in ("norm1", "norm2"):
            tensors.append((f"l{l}.{nm}", hidden))
    tensors.append(("final_norm", hidden))
    tensors.append(("head", vocab * hidden))
    total = sum(t[1] for t in tensors)
    n = total // shard
    segs: List[Segment] = []
    pos = 0
    for nm, ln in tensors:
        if pos >= n:
            break
        take = min(ln, n - pos)
        segs.append((nm, pos, take))
        pos += ln
    return n, segs


def moe_segments(hidden: int, ffn: int, experts: int = 8) -> Tuple[int, List[Segment]]:
    per = 3 * hidden * ffn
    return experts * per, [(f"expert{e}", e * per, per) for e in range(experts)]


def gauss_1m(n: int = 1 << 20) -> Workload:
    return Workload("gauss_1m", "gauss", n, torch.float32, 4, 256, steps=3, num_workers=1,
                    segments=(("all", 0, n),))


def llama7b_shard(bits: int = 4, block_size: int = 256, num_workers: int = 8,
                  hidden: int = 4096, ffn: int = 11008, vocab: int = 32000, layers: int = 32) -> Workload:
    n, segs = llama_segments(hidden, ffn, vocab, layers)
    return Workload(f"llama7b_shard_{bits}bit_b{block_size}", "student_t", n, torch.bfloat16,
                    bits, block_size, num_workers=num_workers, steps=20, segments=tuple(segs))


def mixtral_moe_shard(hidden: int = 4096, ffn: int = 14336, experts: int = 8) -> Workload:
    n, segs = moe_segments(hidden, ffn, experts)
    return Workload("mixtral_moe_shard_4bit_b128", "moe", n, torch.bfloat16, 4, 128,
                    num_workers=1, steps=10, segments=tuple(segs))


def dense70b_shard(n: int = 2_200_000_000, num_workers: int = 16) -> Workload:
    return Workload("dense70b_shard_4bit_b256", "outlier", n, torch.bfloat16, 4, 256,
                    num_workers=num_workers, steps=20, segments=(("all", 0, n),))


ZERO_EXPERTS = (1, 4, 6)


def by_name(name: str) -> Workload:
    """The five benchmark workloads at full size."""
    table = {
        "gauss_1m": gauss_1m,
        "llama7b_shard_4bit_b256": lambda: llama7b_shard(4, 256, 8),
        "llama7b_shard_8bit_b64": lambda: llama7b_shard(8, 64, 8),
        "mixtral_moe_shard_4bit_b128": mixtral_moe_shard,
        "dense70b_shard_4bit_b256": dense70b_shard,
    }
    if name not in table:
        raise KeyError(f"unknown workload {name!r}; known: {sorted(table)}")
    return table[name]()


WORKLOAD_NAMES = ("gauss_1m", "llama7b_shard_4bit_b256", "llama7b_shard_8bit_b64",
                  "mixtral_moe_shard_4bit_b128", "dense70b_shard_4bit_b256")


def small(name: str) -> Workload:
    """Same structure as by_name(name), shrunk so a CPU pass takes well under a second.

    Sizes are chosen to span many tiles and, where the structure allows it, to end
    in a partial block.
    """
    if name == "gauss_1m":
        return gauss_1m(1_000_003).replace(name="gauss_small")
    if name.startswith("llama7b_shard"):
        full = by_name(name)
        w = llama7b_shard(full.bits, full.block_size, full.num_workers,
                          hidden=192, ffn=520, vocab=1500, layers=32)
        return w.replace(name=full.name + "_small", steps=3)
    if name == "mixtral_moe_shard_4bit_b128":
        return mixtral_moe_shard(hidden=96, ffn=344).replace(name=name + "_small", steps=10)
    if name == "dense70b_shard_4bit_b256":
        return dense70b_shard(n=1_500_001, num_workers=16).replace(name=name + "_small", steps=4)
    raise KeyError(name)


def _tensor_factors(w: Workload, lo: float, hi: float) -> List[float]:
    """One log-uniform factor 10^U per tensor; fixed for the workload (not per step)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(BASE_SEED ^ 0x5CA1E)
    u = torch.rand(len(w.segments), generator=g, dtype=torch.float64) * (hi - lo) + lo
    return [10.0 ** float(x) for x in u]


def _chunks(length: int, chunk: int):
    pos = 0
    while pos < length:
        ln = min(chunk, length - pos)
        yield pos, ln
        pos += ln


def gradient(w: Workload, step: int = 0, worker: Optional[int] = None,
             device: str | torch.device = "cpu", chunk: int = 1 << 26) -> torch.Tensor:
    """The flat gradient of `w` for one step (own gradient, or peer `worker`'s)."""
    seed = BASE_SEED + step + (0 if worker is None else 1000 * (worker + 1))
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    out = torch.empty(w.n, dtype=w.grad_dtype, device=dev)

    def randn(k):
        return torch.randn(k, generator=gen, device=dev, dtype=torch.float32)

    if w.recipe == "gauss":
        for pos, ln in _chunks(w.n, chunk):
            out[pos:pos + ln] = (randn(ln) * 1e-3).to(w.grad_dtype)
    elif w.recipe == "student_t":
        factors = _tensor_factors(w, -5.0, -2.0)
        for (_, start, length), fac in zip(w.segments, factors):
            for pos, ln in _chunks(length, chunk):
                z = randn(ln)
                chi = (randn(ln) ** 2 + randn(ln) ** 2 + randn(ln) ** 2) / 3.0
                t = z / torch.sqrt(chi)
                out[start + pos:start + pos + ln] = (t * fac).to(w.grad_dtype)
    elif w.recipe == "moe":
        factors = _tensor_factors(w, -6.0, -3.0)
        for e, ((_, start, length), fac) in enumerate(zip(w.segments, factors)):
            if e in ZERO_EXPERTS:
                out[start:start + length] = 0
                continue
            for pos, ln in _chunks(length, chunk):
                out[start + pos:start + pos + ln] = (randn(ln) * fac).to(w.grad_dtype)
    elif w.recipe == "outlier":
        for pos, ln in _chunks(w.n, chunk):
            z = randn(ln) * 1e-3
            hit = torch.rand(ln, generator=gen, device=dev) < 1e-3
            z = torch.where(hit, z * 100.0, z)
            out[pos:pos + ln] = z.to(w.grad_dtype)
    else:
        raise ValueError(w.recipe)
    return out


def algorithmic_bytes(w: Workload) -> Tuple[float, float]:
    """Bytes the method has to move per element: (compensate-quantize, dequant-reduce).

    compensate-quantize reads the gradient and the state, writes the state, the
    packed codes and one fp32 step per block; dequant-reduce reads W payloads and
    writes one fp32 value.
    """
    gsz = 2 if w.grad_dtype == torch.bfloat16 else 4
    payload = w.bits / 8.0 + 4.0 / w.block_size
    return gsz + 4 + 4 + payload, w.num_workers * payload + 4


def as_numpy_grad(t: torch.Tensor):
    """Host copy in the form the oracle takes: float32, or uint16 bf16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()

