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

Random numbers come from a counter-based generator keyed on (BASE_SEED, step,
worker, tensor, index within the tensor), written in integer operations and table
look-ups so that the CPU and the GPU produce the same bytes (see below).
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


# ---------------------------------------------------------------------------------------
# The random numbers: a counter-based generator, so that every element is a pure function of
# (seed, step, worker, tensor, index within the tensor).  It is written once, in torch
# integer operations and table look-ups plus float64 add/multiply (correctly rounded on every
# device), and therefore gives the same bytes on the CPU and on the GPU, in any chunking.
#
#   bits     x = mix(key + index * GOLDEN), mix = the SplitMix64 finaliser, key = the mix of
#            (seed, step, worker, tensor); two 32-bit draws per element (high and low half)
#   normal   inverse-CDF sampling of |Z| from a table of 2^16 + 1 quantiles with linear
#            interpolation on 15 more bits, the last cell (p > 1 - 2^-16) from a second table
#            of 2^15 quantiles; the sign is one more bit
#   t(3)     the same with Student's t quantiles (3 degrees of freedom)
# The quantile tables are computed once per process on the host (scipy.special, float64) and
# rounded to float32 precision, which makes them insensitive to last-bit differences between
# builds of the special functions; the per-tensor factors 10^U use decimal arithmetic.
# ---------------------------------------------------------------------------------------
_GOLDEN = 0x9E3779B97F4A7C15
_M1, _M2 = 0xBF58476D1CE4E5B9, 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1
_CELLS, _FRAC_BITS = 1 << 16, 15


def _mix_int(x: int) -> int:
    """SplitMix64 finaliser on a Python integer (mod 2^64)."""
    x &= _MASK64
    x = ((x ^ (x >> 30)) * _M1) & _MASK64
    x = ((x ^ (x >> 27)) * _M2) & _MASK64
    return x ^ (x >> 31)


def stream_key(seed: int, step: int, worker: Optional[int], tensor: int) -> int:
    """One 64-bit key per (seed, step, worker, tensor); worker None is this worker's own gradient."""
    k = _mix_int(seed)
    for part in (step, 0 if worker is None else worker + 1, tensor):
        k = _mix_int(k ^ _mix_int(part + 0x632BE59BD9B4E019))
    return k


def _signed(x: int) -> int:
    x &= _MASK64
    return x - (1 << 64) if x >> 63 else x


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right of int64 bit patterns."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def random_bits(key: int, first: int, count: int, device) -> torch.Tensor:
    """int64 bit patterns x_i = mix(key + i * GOLDEN) for i in [first, first + count)."""
    i = torch.arange(first, first + count, dtype=torch.int64, device=device)
    x = i * _signed(_GOLDEN) + _signed(key)          # wraps mod 2^64
    x = (x ^ _lsr(x, 30)) * _signed(_M1)
    x = (x ^ _lsr(x, 27)) * _signed(_M2)
    return x ^ _lsr(x, 31)


_TABLES: dict = {}


def _quantile_tables(kind: str, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """(body, tail): quantiles of |X| at p = i / 2^16, i = 0 .. 2^16 - 1 plus the left edge of the
    last cell repeated, and at the mid-points of the 2^15 sub-cells of the last cell."""
    dev = torch.device(device)
    hit = _TABLES.get((kind, str(dev)))
    if hit is not None:
        return hit
    host = _TABLES.get((kind, "host"))
    if host is None:
        import numpy as np
        from scipy import special
        ppf = special.ndtri if kind == "normal" else (lambda p: special.stdtrit(3.0, p))
        p_body = np.arange(_CELLS, dtype=np.float64) / _CELLS                      # 0 .. 1 - 2^-16
        p_tail = (_CELLS - 1 + (np.arange(1 << _FRAC_BITS, dtype=np.float64) + 0.5) / (1 << _FRAC_BITS)) / _CELLS
        body = ppf(0.5 + p_body / 2)
        body = np.concatenate([body, body[-1:]])                                     # entry 2^16 is never the
        tail = ppf(0.5 + p_tail / 2)                                                 # right end of a used cell
        host = tuple(torch.from_numpy(t.astype(np.float32).astype(np.float64)) for t in (body, tail))
        _TABLES[(kind, "host")] = host
    out = tuple(t.to(dev) for t in host)
    _TABLES[(kind, str(dev))] = out
    return out


def _symmetric_from_bits(u32: torch.Tensor, kind: str) -> torch.Tensor:
    """float64 samples of a symmetric distribution from 32-bit draws (int64 tensor, values < 2^32)."""
    body, tail = _quantile_tables(kind, u32.device)
    cell = (u32 >> 16) & (_CELLS - 1)
    frac = (u32 >> 1) & ((1 << _FRAC_BITS) - 1)
    lo = body[cell]
    hi = body[cell + 1]
    t = (frac.to(torch.float64) + 0.5) * (1.0 / (1 << _FRAC_BITS))                   # exact
    mag = lo + (hi - lo) * t
    mag = torch.where(cell == _CELLS - 1, tail[frac], mag)
    return torch.where((u32 & 1) == 1, -mag, mag)


def _hi32(x: torch.Tensor) -> torch.Tensor:
    return _lsr(x, 32)


def _lo32(x: torch.Tensor) -> torch.Tensor:
    return x & 0xFFFFFFFF


def _tensor_factors(w: Workload, lo: float, hi: float) -> List[float]:
    """One log-uniform factor 10^U per tensor; fixed for the workload (not per step)."""
    import decimal
    out = []
    with decimal.localcontext() as ctx:
        ctx.prec = 40
        for t in range(len(w.segments)):
            h = _mix_int(stream_key(BASE_SEED ^ 0x5CA1E, 0, None, t)) >> 11           # 53 uniform bits
            u = decimal.Decimal(lo) + (decimal.Decimal(hi) - decimal.Decimal(lo)) * decimal.Decimal(h) / decimal.Decimal(1 << 53)
            out.append(float(decimal.Decimal(10) ** u))
    return out


def _chunks(length: int, chunk: int):
    pos = 0
    while pos < length:
        ln = min(chunk, length - pos)
        yield pos, ln
        pos += ln


OUTLIER_THRESHOLD = 4294967          # floor(1e-3 * 2^32): an element is an outlier when its low draw is below


def gradient(w: Workload, step: int = 0, worker: Optional[int] = None,
             device: str | torch.device = "cpu", chunk: int = 1 << 24) -> torch.Tensor:
    """The flat gradient of `w` for one step (own gradient, or peer `worker`'s).  The same bytes
    on every device and for every chunk size."""
    dev = torch.device(device)
    out = torch.empty(w.n, dtype=w.grad_dtype, device=dev)

    def store(start, values64):
        out[start:start + values64.numel()] = values64.to(torch.float32).to(w.grad_dtype)

    if w.recipe == "student_t":
        factors = _tensor_factors(w, -5.0, -2.0)
    elif w.recipe == "moe":
        factors = _tensor_factors(w, -6.0, -3.0)
    else:
        factors = [1e-3] * len(w.segments)
    for t, ((_, start, length), fac) in enumerate(zip(w.segments, factors)):
        if w.recipe == "moe" and t in ZERO_EXPERTS:
            out[start:start + length] = 0
            continue
        key = stream_key(BASE_SEED, step, worker, t)
        for pos, ln in _chunks(length, chunk):
            x = random_bits(key, pos, ln, dev)
            if w.recipe in ("gauss", "moe"):
                v = _symmetric_from_bits(_hi32(x), "normal") * fac
            elif w.recipe == "student_t":
                v = _symmetric_from_bits(_hi32(x), "student_t3") * fac
            elif w.recipe == "outlier":
                v = _symmetric_from_bits(_hi32(x), "normal") * fac
                v = torch.where(_lo32(x) < OUTLIER_THRESHOLD, v * 100.0, v)
            else:
                raise ValueError(w.recipe)
            store(start + pos, v)
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

