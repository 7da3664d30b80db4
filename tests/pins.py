"""Checks that pin the CPU oracle to what the paper and arithmetic fix.

Each check takes a loaded oracle library handle, so the same checks can be run
on the real oracle (they must pass) and on copies with a planted mistake (at
least one must fail; see test_oracle_mutants.py).  Nothing here calls the GPU.

Citations are to LoCo, arXiv 2407.04480.
"""
from __future__ import annotations

import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
FLT_MIN = np.float32(np.finfo(np.float32).tiny)


# ---------------------------------------------------------------- helpers
def unpack(codes: np.ndarray, n: int, bits: int) -> np.ndarray:
    """Integer codes from packed bytes (int8, or two's complement nibbles, low first)."""
    if bits == 8:
        return codes[:n].view(np.int8).astype(np.int64)
    nib = np.empty(2 * codes.size, dtype=np.int64)
    nib[0::2] = codes & 15
    nib[1::2] = codes >> 4
    nib = nib[:n]
    return np.where(nib >= 8, nib - 16, nib)


def qrange(bits):
    return -(1 << (bits - 1)), (1 << (bits - 1)) - 1


def block_index(n, B):
    return np.arange(n) // B


def rng_grad(rng, n, kind="normal", scale=1e-3):
    if kind == "normal":
        g = rng.standard_normal(n) * scale
    elif kind == "student":
        g = rng.standard_t(3, n) * scale
    elif kind == "uniform":
        g = rng.uniform(-scale, scale, n)
    elif kind == "wide":  # magnitudes over many binades
        g = rng.standard_normal(n) * np.exp2(rng.integers(-40, 10, n))
    else:
        raise ValueError(kind)
    return g.astype(np.float32)


def to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest even (input-making helper)."""
    u = x32.view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def cq(lib, g, e, bits, B, beta, reset=0, threads=1):
    return oracle.compensate_quantize(g, e, bits, B, beta, reset, threads=threads, lib=lib)


def decode1(lib, codes, scales, n, bits, B):
    return oracle.dequant_reduce(codes, scales, 1, n, bits, B, lib=lib)


def ulp32(x):
    x = np.abs(x.astype(np.float32))
    return np.spacing(x).astype(np.float64)


# ---------------------------------------------------------------- the pins
def check_worked_example(lib):
    """Hand-derived dyadic two-step example (Alg. 1 steps 1-2; Eq. 1-5)."""
    rows = {}
    with open(os.path.join(GOLDEN, "worked_example_p4_b8.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rows[key] = vals
    unit = 2.0 ** int(rows["unit_log2"][0])
    bits, B, beta = int(rows["bits"][0]), int(rows["block"][0]), float(rows["beta"][0])
    vec = lambda k: (np.array([float(v) for v in rows[k]]) * unit).astype(np.float32)
    g = vec("g")
    e = np.zeros_like(g)
    oracle.error_state_init(e, lib=lib)
    for step, nxt in ((0, "e1"), (1, "e2")):
        if step == 1:
            assert np.array_equal((g + e), vec("h1"))
        codes, scales = cq(lib, g, e, bits, B, beta)
        want_bytes = np.array([int(b, 16) for b in rows[f"bytes{step}"]], dtype=np.uint8)
        assert np.array_equal(codes, want_bytes), (step, codes, want_bytes)
        assert np.array_equal(unpack(codes, g.size, bits), [int(v) for v in rows[f"q{step}"]])
        assert scales.tolist() == [float(rows[f"scale{step}"][0]) * unit]
        assert np.array_equal(e, vec(nxt)), (step, e / unit)


def check_exact_reconstruction(lib):
    """Eq. 4: d + delta = h.  With beta = 1 the new state is delta itself."""
    rng = np.random.default_rng(101)
    for bits, B, kind in ((4, 256, "normal"), (8, 64, "student"), (4, 128, "wide"), (8, 32, "uniform")):
        n = 40 * B + 17
        g = rng_grad(rng, n, kind)
        e0 = rng_grad(rng, n, "normal", 2e-4)
        h = g + e0                                     # Eq. 2 in binary32
        e = e0.copy()
        codes, scales = cq(lib, g, e, bits, B, 1.0)
        delta = e
        d = decode1(lib, codes, scales, n, bits, B)
        back = (d + delta).astype(np.float32)
        # h - d is exact (Sterbenz) when d == 0 or d/2 <= h <= 2d; the only other case is
        # |q| = 1 with |h| a hair under half a step, where one rounding may remain.
        with np.errstate(divide="ignore", invalid="ignore"):
            ratio = np.where(d != 0, h.astype(np.float64) / d.astype(np.float64), 1.0)
        safe = (d == 0) | ((ratio >= 0.5) & (ratio <= 2.0))
        assert np.array_equal(back[safe], h[safe])
        rest = ~safe
        assert rest.mean() < 1e-3
        assert np.all(np.abs(unpack(codes, n, bits)[rest]) == 1)
        assert np.all(np.abs(back[rest].astype(np.float64) - h[rest]) <= ulp32(h[rest]))


def check_rounding_bound(lib):
    """Lemma 5 with 1/s = D_b: |h - C(h)| <= D_b/2 (plus the rounding of r_b and h*r_b);
    the block's largest element gets code +-qmax; no code reaches -2^(p-1)."""
    rng = np.random.default_rng(202)
    for bits, B in ((4, 256), (8, 64), (4, 64), (8, 256)):
        qmin, qmax = qrange(bits)
        n = 64 * B + 5
        g = rng_grad(rng, n, "student")
        e0 = rng_grad(rng, n, "normal", 1e-4)
        h = g + e0
        e = e0.copy()
        codes, scales = cq(lib, g, e, bits, B, 1.0)
        q = unpack(codes, n, bits)
        D = scales[block_index(n, B)].astype(np.float64)
        assert np.all(np.abs(e) <= D * (0.5 + 4 * qmax * 2.0 ** -24))
        assert q.min() >= -qmax and q.max() <= qmax
        nb = oracle.num_blocks(n, B)
        for b in range(nb):
            sl = slice(b * B, min(n, (b + 1) * B))
            i = np.argmax(np.abs(h[sl]))
            assert abs(q[sl][i]) == qmax
            assert np.sign(q[sl][i]) == np.sign(h[sl][i])
            # the stored step is max|h|/qmax, one binary32 division
            assert scales[b] == np.float32(np.abs(h[sl]).max()) / np.float32(qmax)


def check_ema_recurrence(lib):
    """Eq. 5 unrolled: e~_K = beta * sum_k (1-beta)^(K-1-k) delta_k with e~_0 = 0."""
    rng = np.random.default_rng(303)
    for beta in (0.25, 0.5, 0.9):
        bits, B, n, K = 4, 64, 64 * 30 + 9, 7
        e = np.ones(n, dtype=np.float32)
        oracle.error_state_init(e, lib=lib)
        assert not e.any()
        deltas = []
        for k in range(K):
            g = rng_grad(rng, n, "normal")
            h = g.astype(np.float64) + e.astype(np.float64)
            codes, scales = cq(lib, g, e, bits, B, beta)
            d = decode1(lib, codes, scales, n, bits, B).astype(np.float64)
            deltas.append(h - d)
        closed = np.zeros(n)
        for k, dl in enumerate(deltas):
            closed += beta * (1.0 - beta) ** (K - 1 - k) * dl
        tol = K * 2.0 ** -22 * max(np.abs(dl).max() for dl in deltas)
        assert np.abs(e - closed).max() <= tol
        assert np.abs(closed).max() > 100 * tol          # the check has teeth


def check_beta_special_cases(lib):
    """beta = 1 is classic error feedback (Eq. 4); beta = 0 keeps e~ = 0 for ever."""
    rng = np.random.default_rng(404)
    bits, B, n = 4, 128, 128 * 20 + 3
    g0, g1 = rng_grad(rng, n), rng_grad(rng, n)
    # beta = 0: the state stays zero and codes are those of a fresh state
    e = np.zeros(n, np.float32)
    c0, s0 = cq(lib, g0, e, bits, B, 0.0)
    assert not e.any()
    c1, s1 = cq(lib, g1, e, bits, B, 0.0)
    assert not e.any()
    f = np.zeros(n, np.float32)
    c1f, s1f = cq(lib, g1, f, bits, B, 0.7)
    assert np.array_equal(c1, c1f) and np.array_equal(s1, s1f)
    # beta = 1: the state equals h - d exactly
    e = np.zeros(n, np.float32)
    cq(lib, g0, e, bits, B, 1.0)
    h = g1 + e
    c, s = cq(lib, g1, e, bits, B, 1.0)
    d = decode1(lib, c, s, n, bits, B)
    assert np.array_equal(e, (h - d).astype(np.float32))
    # a general beta: one step from a known state, against Eq. 5 written in binary64
    e0 = rng_grad(rng, n, "normal", 3e-4)
    e = e0.copy()
    beta = 0.3
    c, s = cq(lib, g0, e, bits, B, beta)
    d = decode1(lib, c, s, n, bits, B).astype(np.float64)
    h = (g0 + e0).astype(np.float64)
    want = (1.0 - np.float64(np.float32(beta))) * e0 + np.float64(np.float32(beta)) * (h - d)
    assert np.abs(e - want).max() <= 2.0 ** -22 * np.abs(want).max()


def check_zero_error_fixed_point(lib):
    """Eq. 1 on exactly representable input: h = m * 2^-t, |m| <= qmax, some |m| = qmax
    in every block  =>  D = 2^-t, q = m, delta = 0, the state stays exactly 0."""
    rng = np.random.default_rng(505)
    for bits, B, t in ((4, 256, 19), (8, 64, 17), (4, 128, 10), (8, 256, 30)):
        qmin, qmax = qrange(bits)
        n = 33 * B
        e = np.zeros(n, np.float32)
        for _ in range(3):
            m = rng.integers(-qmax, qmax + 1, n)
            pos = np.arange(0, n, B) + rng.integers(0, B, n // B)
            m[pos] = rng.choice([-qmax, qmax], n // B)
            g = (m * 2.0 ** -t).astype(np.float32)
            codes, scales = cq(lib, g, e, bits, B, 0.25)
            assert np.array_equal(unpack(codes, n, bits), m)
            assert np.all(scales == np.float32(2.0 ** -t))
            assert not e.any()
            assert np.array_equal(decode1(lib, codes, scales, n, bits, B), g)


def check_brute_force_levels(lib):
    """Eq. 1: q is the level of [-2^(p-1), 2^(p-1)-1] nearest to h*s (ties to even),
    found here by trying every level in binary64."""
    rng = np.random.default_rng(606)
    flips = total = 0
    for trial in range(1500):
        bits = (4, 8)[trial & 1]
        qmin, qmax = qrange(bits)
        B = int(rng.choice([8, 16, 32, 64]))
        n = int(rng.integers(1, 65))
        g = rng_grad(rng, n, ("normal", "student", "wide")[trial % 3])
        e0 = rng_grad(rng, n, "normal", 1e-4) if trial % 5 else np.zeros(n, np.float32)
        h = g + e0
        e = e0.copy()
        codes, scales = cq(lib, g, e, bits, B, 1.0)
        q = unpack(codes, n, bits)
        levels = np.arange(qmin, qmax + 1, dtype=np.float64)
        for b in range(oracle.num_blocks(n, B)):
            sl = slice(b * B, min(n, (b + 1) * B))
            D = np.float32(np.abs(h[sl]).max()) / np.float32(qmax)
            if D < FLT_MIN:
                assert scales[b] == 0 and not q[sl].any()
                continue
            assert scales[b] == D
            x = h[sl].astype(np.float64) / np.float64(D)
            dist = np.abs(x[:, None] - levels[None, :])
            best = dist.min(axis=1)
            cand = dist <= best[:, None]                       # one level, or two at a tie
            ok = cand[np.arange(x.size), q[sl] - qmin]
            tie = cand.sum(axis=1) == 2
            even_ok = ~tie | (q[sl] % 2 == 0)
            near_half = np.abs(np.abs(x - np.floor(x)) - 0.5) <= 4 * qmax * 2.0 ** -24
            bad = ~(ok & even_ok)
            assert not np.any(bad & ~near_half), (trial, b)
            # even when the binary32 rounding of s_b moved a near-tie, the code is adjacent
            assert np.all(np.abs(q[sl] - x) <= 0.5 + 4 * qmax * 2.0 ** -24)
            flips += int(bad.sum())
            total += x.size
    assert flips <= 1e-3 * total


def check_telescoping(lib):
    """Lemma 1 with an uncompressed state: d_k = g_k + (e~_k - e~_{k+1})/beta, hence
    sum_k d_k = sum_k g_k - e~_K / beta."""
    rng = np.random.default_rng(707)
    for bits, B, beta, K in ((4, 256, 0.25, 10), (8, 64, 0.5, 20), (4, 128, 1.0, 10)):
        n = B * 12 + 1
        e = np.zeros(n, np.float32)
        sum_d = np.zeros(n)
        sum_g = np.zeros(n)
        gmax = 0.0
        for _ in range(K):
            g = rng_grad(rng, n, "normal")
            codes, scales = cq(lib, g, e, bits, B, beta)
            sum_d += decode1(lib, codes, scales, n, bits, B)
            sum_g += g
            gmax = max(gmax, float(np.abs(g).max()))
        beta32 = np.float64(np.float32(beta))
        assert np.abs(sum_d - (sum_g - e / beta32)).max() <= K * 2.0 ** -21 * gmax / beta32
        assert np.abs(sum_d - sum_g).max() > 20 * K * 2.0 ** -21 * gmax / beta32  # non-trivial


def check_fixed_scale_form(lib):
    """Eq. 1 literally, at the paper's s = 2^19 (4-bit) and s = 2^17: when a block's
    largest |h| is qmax/s the block scale is s exactly and q = clip(rint(h*s))."""
    rng = np.random.default_rng(808)
    for bits, B, log2s in ((4, 256, 19), (4, 64, 17), (8, 64, 19), (8, 128, 17)):
        qmin, qmax = qrange(bits)
        s = np.float32(2.0 ** log2s)
        n = 50 * B
        top = np.float32(qmax) / s
        g = rng.uniform(-float(top), float(top), n).astype(np.float32)
        e0 = np.zeros(n, np.float32)
        pos = np.arange(0, n, B) + rng.integers(0, B, n // B)
        g[pos] = top * rng.choice([-1.0, 1.0], n // B).astype(np.float32)
        e = e0.copy()
        codes, scales = cq(lib, g, e, bits, B, 1.0)
        assert np.all(scales == np.float32(1.0) / s)
        want = np.clip(np.rint(g * s), qmin, qmax).astype(np.int64)   # power-of-two product: exact
        assert np.array_equal(unpack(codes, n, bits), want)
        # decompressor: float(q)/s, and Eq. 4
        d = decode1(lib, codes, scales, n, bits, B)
        assert np.array_equal(d, (want / float(s)).astype(np.float32))
        assert np.array_equal(e, g - d)


def check_reset(lib):
    """e~_0 = 0; Eq. 7: on a reset step the payload is that of the old state and the
    new state is all zeros."""
    rng = np.random.default_rng(909)
    bits, B, n = 4, 256, 256 * 9 + 100
    g = rng_grad(rng, n)
    e0 = rng_grad(rng, n, "normal", 2e-4)
    ea, eb = e0.copy(), e0.copy()
    ca, sa = cq(lib, g, ea, bits, B, 0.25, reset=0)
    cb, sb = cq(lib, g, eb, bits, B, 0.25, reset=1)
    assert np.array_equal(ca, cb) and np.array_equal(sa, sb)
    assert ea.any() and not eb.any()
    assert np.all(np.signbit(eb) == False)  # noqa: E712


def check_reset_schedule(lib):
    """Eq. 7 / Alg. 1 as printed: the state written by step k is zero exactly when k % T_c = 0,
    i.e. at k = 0, T_c, 2 T_c, ... (T_c = 512 or 1024 in Sec. 3.2); composed with the step itself,
    the state after a reset step is zero and the steps between resets follow Eq. 5."""
    for T in (2, 3, 7, 128, 512, 1024):
        got = [k for k in range(0, 3 * T + 2) if lib.loco_ref_reset_due(k, T)]
        assert got == [0, T, 2 * T, 3 * T], (T, got)
    assert all(lib.loco_ref_reset_due(k, 1) for k in range(0, 10))
    assert not any(lib.loco_ref_reset_due(k, 0) for k in range(0, 2000))
    assert not any(lib.loco_ref_reset_due(k, -4) for k in range(0, 20))
    assert lib.loco_ref_reset_due(1 << 40, 1 << 20) and not lib.loco_ref_reset_due((1 << 40) + 1, 1 << 20)
    assert lib.loco_ref_reset_due(3 * ((1 << 33) + 1), (1 << 33) + 1)
    # composed with the step: T_c = 3 over 8 steps, beta = 1 makes the state the raw error of the step
    rng = np.random.default_rng(77)
    bits, B, n, T = 4, 64, 64 * 5 + 9, 3
    e = np.zeros(n, np.float32)
    for k in range(8):
        g = rng_grad(rng, n)
        h = g + e
        due = lib.loco_ref_reset_due(k, T)
        codes, scales = cq(lib, g, e, bits, B, 1.0, reset=due)
        if k % T == 0:
            assert due and not e.any()
        else:
            assert not due
            d = decode1(lib, codes, scales, n, bits, B)
            assert np.array_equal(e, h - d)


def check_dequant_reduce(lib):
    """Eq. 8: N = 1 returns float(q)/s; N equal payloads return that value again (exactly
    for N = 2); a general N is the mean of the decoded payloads."""
    rng = np.random.default_rng(1010)
    for bits, B in ((4, 256), (8, 64)):
        n = B * 20 + 7
        nb, cb = oracle.num_blocks(n, B), oracle.code_bytes(n, bits)
        payloads = []
        for w in range(5):
            e = np.zeros(n, np.float32)
            payloads.append(cq(lib, rng_grad(rng, n, "student"), e, bits, B, 0.25))
        dec = [unpack(c, n, bits).astype(np.float32) * s[block_index(n, B)] for c, s in payloads]
        c0, s0 = payloads[0]
        assert np.array_equal(decode1(lib, c0, s0, n, bits, B), dec[0])
        for W in (2, 4, 8, 16):
            out = oracle.dequant_reduce(np.tile(c0, W), np.tile(s0, W), W, n, bits, B, lib=lib)
            if W == 2:      # x + x is exact, and so is the halving
                assert np.array_equal(out, dec[0])
            else:           # 3x, 5x, ... round: one ulp per addition at most
                assert np.all(np.abs(out.astype(np.float64) - dec[0]) <= W * ulp32(dec[0]))
        # strided layout with padding between payloads, W = 3 and 5
        cstride, sstride = cb + 13, nb + 3
        for W in (3, 5):
            codes = np.zeros(W * cstride, np.uint8)
            scales = np.zeros(W * sstride, np.float32)
            for w in range(W):
                codes[w * cstride:w * cstride + cb] = payloads[w][0]
                scales[w * sstride:w * sstride + nb] = payloads[w][1]
            out = oracle.dequant_reduce(codes, scales, W, n, bits, B, cstride, sstride, lib=lib)
            mean = np.mean(np.stack(dec[:W]).astype(np.float64), axis=0)
            top = np.abs(np.stack(dec[:W])).max(axis=0)
            assert np.all(np.abs(out - mean) <= (W + 1) * 2.0 ** -24 * top)
            assert np.abs(mean).max() > 0
        # order of the workers: at most (W-1) ulp of the largest partial sum
        W = 5
        codes = np.concatenate([p[0] for p in payloads])
        scales = np.concatenate([p[1] for p in payloads])
        fwd = oracle.dequant_reduce(codes, scales, W, n, bits, B, lib=lib)
        rcodes = np.concatenate([p[0] for p in payloads[::-1]])
        rscales = np.concatenate([p[1] for p in payloads[::-1]])
        rev = oracle.dequant_reduce(rcodes, rscales, W, n, bits, B, lib=lib)
        bound = (W - 1) * ulp32(np.abs(np.stack(dec)).sum(axis=0).astype(np.float32))
        assert np.all(np.abs(fwd.astype(np.float64) - rev) <= bound)


def check_bf16_widening(lib):
    """A bf16 gradient is widened exactly: same result as the same values given as fp32."""
    rng = np.random.default_rng(1111)
    bits, B, n = 4, 64, 64 * 11 + 3
    gb = to_bf16_bits(rng_grad(rng, n, "student"))
    g32 = bf16_bits_to_f32(gb)
    e0 = rng_grad(rng, n, "normal", 1e-4)
    ea, eb = e0.copy(), e0.copy()
    ca, sa = cq(lib, gb, ea, bits, B, 0.25)
    cb, sb = cq(lib, g32, eb, bits, B, 0.25)
    assert np.array_equal(ca, cb) and np.array_equal(sa, sb) and np.array_equal(ea, eb)
    assert sa.any()


def check_edges(lib):
    """Empty input, one element, odd length (last high nibble 0), partial last block,
    all-zero and subnormal-step blocks (stored step +0, zero codes, error keeps h)."""
    e = np.zeros(0, np.float32)
    c, s = cq(lib, np.zeros(0, np.float32), e, 4, 256, 0.25)
    assert c.size == 0 and s.size == 0
    assert oracle.dequant_reduce(c, s, 3, 0, 4, 256, lib=lib).size == 0
    # one element: it is its own block maximum
    for bits in (4, 8):
        qmin, qmax = qrange(bits)
        e = np.zeros(1, np.float32)
        c, s = cq(lib, np.array([-0.3], np.float32), e, bits, 256, 1.0)
        assert unpack(c, 1, bits).tolist() == [-qmax] and c.size == 1
        assert s[0] == np.float32(0.3) / np.float32(qmax)
    # odd n, 4-bit: the unused high nibble is zero
    rng = np.random.default_rng(1212)
    n = 2 * 64 + 37
    g = rng_grad(rng, n)
    e = np.zeros(n, np.float32)
    c, s = cq(lib, g, e, 4, 64, 0.25)
    assert c.size == (n + 1) // 2 and (c[-1] >> 4) == 0 and s.size == 3
    # the partial last block sees only its own elements
    tail = g[128:]
    et = np.zeros(tail.size, np.float32)
    ct, st = cq(lib, tail, et, 4, 64, 0.25)
    assert st[0] == s[2] and np.array_equal(ct, c[64:]) and np.array_equal(et, e[128:])
    # zero block between live blocks; a block whose step would be subnormal
    B = 64
    g = rng_grad(rng, 4 * B)
    g[B:2 * B] = 0
    tiny = np.float32(2.0 ** -127)                    # max|h|/7 < FLT_MIN
    g[2 * B:3 * B] = (rng.uniform(-1, 1, B) * tiny).astype(np.float32)
    e = np.zeros(4 * B, np.float32)
    c, s = cq(lib, g, e, 4, B, 1.0)
    q = unpack(c, 4 * B, 4)
    assert s[1] == 0 and not np.signbit(s[1]) and s[2] == 0 and s[0] > 0 and s[3] > 0
    assert not q[B:3 * B].any() and q[:B].any() and q[3 * B:].any()
    assert np.array_equal(e[B:3 * B], g[B:3 * B])
    # smallest live step: max|h| = 7 * FLT_MIN
    g = np.zeros(B, np.float32)
    g[3] = np.float32(7) * FLT_MIN
    g[5] = np.float32(-3) * FLT_MIN
    e = np.zeros(B, np.float32)
    c, s = cq(lib, g, e, 4, B, 1.0)
    assert s[0] == FLT_MIN and unpack(c, B, 4)[[3, 5]].tolist() == [7, -3] and not e.any()


def check_threads_agree(lib):
    """The threaded driver only splits ranges: same bytes as one thread."""
    rng = np.random.default_rng(1313)
    for bits, B, n in ((4, 256, 256 * 37 + 11), (8, 64, 64 * 101 + 63), (4, 7, 1001)):
        g = rng_grad(rng, n, "student")
        e0 = rng_grad(rng, n, "normal", 1e-4)
        ea, eb = e0.copy(), e0.copy()
        ca, sa = cq(lib, g, ea, bits, B, 0.25)
        cb, sb = cq(lib, g, eb, bits, B, 0.25, threads=5)
        assert np.array_equal(ca, cb) and np.array_equal(sa, sb) and np.array_equal(ea, eb)
        W = 3
        out1 = oracle.dequant_reduce(np.tile(ca, W), np.tile(sa, W), W, n, bits, B, lib=lib)
        out5 = oracle.dequant_reduce(np.tile(ca, W), np.tile(sa, W), W, n, bits, B, threads=5, lib=lib)
        assert np.array_equal(out1, out5)


ALL_CHECKS = [
    check_worked_example,
    check_exact_reconstruction,
    check_rounding_bound,
    check_ema_recurrence,
    check_beta_special_cases,
    check_zero_error_fixed_point,
    check_brute_force_levels,
    check_telescoping,
    check_fixed_scale_form,
    check_reset,
    check_reset_schedule,
    check_dequant_reduce,
    check_bf16_widening,
    check_edges,
    check_threads_agree,
]


# ======================================================================================
# The paper's literal form: global scale s, 8-bit error state with scale s_e (Alg. 1 as
# printed; Eq. 1-3, 5, 7, 8).  Oracle: loco_ref_fixed_*.
# ======================================================================================
def fcq(lib, g, e8, bits, log2_s, se_mult, beta, reset=0, threads=1):
    return oracle.fixed_compensate_quantize(g, e8, bits, log2_s, se_mult, beta, reset, threads=threads, lib=lib)


def near_tie(x, rel=2.0 ** -21, tiny=1e-30):
    """x (float64 shadow of a binary32 product) so close to k + 1/2 that binary32 may round it either way."""
    return np.abs(np.abs(x - np.floor(x)) - 0.5) <= np.abs(x) * rel + tiny


def check_fixed_worked_example(lib):
    """Hand-derived dyadic example of Alg. 1 as printed (Eq. 1-3, 5, 7, 8)."""
    rows = {}
    with open(os.path.join(GOLDEN, "worked_example_fixed_scale_p4.txt")) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                key, *vals = line.split()
                rows[key] = vals
    bits, log2_s, mult, beta = int(rows["bits"][0]), int(rows["log2_s"][0]), int(rows["se_mult"][0]), float(rows["beta"][0])
    g = np.array([float(v) for v in rows["g"]], np.float32)
    ints = lambda k: [int(v) for v in rows[k]]
    e8 = np.zeros(g.size, np.int8)
    payloads = []
    for step in (0, 1):
        codes = fcq(lib, g, e8, bits, log2_s, mult, beta)
        want = np.array([int(b, 16) for b in rows[f"bytes{step}"]], np.uint8)
        assert np.array_equal(codes, want), (step, codes, want)
        assert unpack(codes, g.size, bits).tolist() == ints(f"q{step}")
        assert e8.tolist() == ints(f"e{step + 1}"), (step, e8)
        payloads.append(codes)
    out = oracle.fixed_dequant_reduce(np.concatenate(payloads), 2, g.size, bits, log2_s, lib=lib)
    assert out.tolist() == [float(v) for v in rows["mean"]]


def check_fixed_nearest_levels(lib):
    """Eq. 1 for the gradient codes and Eq. 7 for the state codes: each is the level of its
    p-bit range nearest to x*s resp. e~'*s_e (binary64 shadow; near-ties whitelisted), and
    the compression error obeys Lemma 5: at most 1/(2s) unless the clamp fired."""
    rng = np.random.default_rng(2024)
    odd = tot = 0
    for trial in range(300):
        bits = (4, 8)[trial & 1]
        qmin, qmax = qrange(bits)
        log2_s = int(rng.choice([19, 17, 10, 3]))
        mult = int(rng.choice([4, 6]))
        beta = float(rng.choice([0.25, 0.5, 1.0, 0.3, 0.9]))
        s, se = 2.0 ** log2_s, mult * 2.0 ** log2_s
        n = int(rng.integers(1, 200))
        g = (rng.standard_normal(n) * rng.choice([0.3, 1, 3, 30]) * qmax / s).astype(np.float32)
        e0 = rng.integers(-128, 128, n).astype(np.int8) if trial % 3 else np.zeros(n, np.int8)
        e8 = e0.copy()
        codes = fcq(lib, g, e8, bits, log2_s, mult, beta)
        q = unpack(codes, n, bits)
        e_hat = e0.astype(np.float64) / se
        h = g.astype(np.float64) + e_hat
        x = h * s
        want_q = np.clip(np.rint(x), qmin, qmax)
        bad = (q != want_q) & ~near_tie(x)
        assert not bad.any(), (trial, x[bad], q[bad])
        assert np.all(np.abs(q - np.clip(x, qmin, qmax)) <= 0.5 + np.abs(x) * 2.0 ** -21)
        unsat = np.abs(x) <= qmax + 0.5
        d = q / s
        assert np.all(np.abs(h - d)[unsat] <= (0.5 + np.abs(x[unsat]) * 2.0 ** -21) / s)      # Lemma 5
        sat = ~unsat & (np.abs(x) > qmax + 1)
        assert np.all(q[sat & (x > 0)] == qmax) and np.all(q[sat & (x < 0)] == qmin)
        b32 = np.float64(np.float32(beta))
        e_new = (1.0 - b32) * e_hat + b32 * (h - d)                                              # Eq. 5
        y = e_new * se
        want_e = np.clip(np.rint(y), -128, 127)
        # the binary32 rounding of e~' moves y by up to |y| 2^-22: near-ties may go either way
        bad_e = (e8 != want_e) & ~near_tie(y, rel=2.0 ** -20)
        assert not bad_e.any(), (trial, y[bad_e], e8[bad_e])
        odd += int(((q != want_q) | (e8 != want_e)).sum())
        tot += 2 * n
    assert odd <= 2e-3 * tot


def check_fixed_zero_error_fixed_point(lib):
    """g = m/s with integer m in range: q = m, delta = 0, the state stays 0 (Eq. 1, 5)."""
    rng = np.random.default_rng(31)
    for bits, log2_s, mult in ((4, 19, 4), (4, 17, 6), (8, 19, 6)):
        qmin, qmax = qrange(bits)
        n = 1001
        e8 = np.zeros(n, np.int8)
        for _ in range(3):
            m = rng.integers(qmin, qmax + 1, n)
            g = (m * 2.0 ** -log2_s).astype(np.float32)
            codes = fcq(lib, g, e8, bits, log2_s, mult, 0.25)
            assert np.array_equal(unpack(codes, n, bits), m)
            assert not e8.any()
            assert np.array_equal(oracle.fixed_dequant_reduce(codes, 1, n, bits, log2_s, lib=lib), g)


def check_fixed_telescoping(lib):
    """Lemma 1 with the compressed state: d_k = g_k + (e^_k - e~_{k+1})/beta, so summed over K
    steps |sum d - sum g + e^_K/beta| <= K/(2 s_e beta): only the state's own rounding is left."""
    rng = np.random.default_rng(47)
    for bits, log2_s, mult, beta, K in ((4, 19, 4, 0.5, 12), (4, 17, 6, 0.25, 20), (8, 19, 6, 1.0, 8)):
        qmin, qmax = qrange(bits)
        s, se = 2.0 ** log2_s, mult * 2.0 ** log2_s
        n = 4000
        e8 = np.zeros(n, np.int8)
        sum_d, sum_g = np.zeros(n), np.zeros(n)
        for _ in range(K):
            g = (rng.uniform(-(qmax - 1), qmax - 1, n) / s).astype(np.float32)   # never clamps
            codes = fcq(lib, g, e8, bits, log2_s, mult, beta)
            sum_d += unpack(codes, n, bits) / s
            sum_g += g
        assert np.abs(e8).max() < 127
        resid = np.abs(sum_d - sum_g + (e8 / se) / beta)
        assert resid.max() <= K / (2 * se * beta) * (1 + 1e-3)
        # and the uncompensated error of one step, 1/(2s), would have added up to far more
        assert np.abs(sum_d - sum_g).max() <= (0.5 / s + 0.5 / se) / beta + K / (2 * se * beta)


def check_fixed_beta_and_reset(lib):
    """beta = 0: re-compressing the decoded state gives the same codes back (the state is
    constant); beta = 1: e' = compressor(h - d; s_e); reset (Eq. 7): same payload, state 0."""
    rng = np.random.default_rng(53)
    bits, log2_s = 4, 19
    s = 2.0 ** log2_s
    n = 3001
    g = (rng.standard_normal(n) * 5 / s).astype(np.float32)
    for mult in (4, 6):
        e0 = rng.integers(-128, 128, n).astype(np.int8)
        e8 = e0.copy()
        c0 = fcq(lib, g, e8, bits, log2_s, mult, 0.0)
        assert np.array_equal(e8, e0)
        ea, eb = e0.copy(), e0.copy()
        ca = fcq(lib, g, ea, bits, log2_s, mult, 0.25, reset=0)
        cb = fcq(lib, g, eb, bits, log2_s, mult, 0.25, reset=1)
        assert np.array_equal(ca, cb) and np.array_equal(ca, c0) and ea.any() and not eb.any()
        e1 = e0.copy()
        c1 = fcq(lib, g, e1, bits, log2_s, mult, 1.0)
        h = g.astype(np.float64) + e0 / (mult * s)
        y = (h - unpack(c1, n, bits) / s) * mult * s
        ok = (e1 == np.clip(np.rint(y), -128, 127)) | near_tie(y, rel=2.0 ** -20)
        assert ok.all()


def check_fixed_matches_block_form(lib):
    """With a zero state and every block's largest |g| equal to qmax/s, the block-scaled
    compressor has scale s exactly, so both forms of Eq. 1 must emit the same codes."""
    rng = np.random.default_rng(59)
    for bits, log2_s, B in ((4, 19, 256), (8, 17, 64)):
        qmin, qmax = qrange(bits)
        s = 2.0 ** log2_s
        n = 20 * B
        g = (rng.uniform(-qmax, qmax, n) / s).astype(np.float32)
        g[np.arange(0, n, B) + rng.integers(0, B, n // B)] = np.float32(qmax / s)
        c_fixed = fcq(lib, g, np.zeros(n, np.int8), bits, log2_s, 4, 0.25)
        c_block, scales = cq(lib, g, np.zeros(n, np.float32), bits, B, 0.25)
        assert np.all(scales == np.float32(1.0 / s))
        assert np.array_equal(c_fixed, c_block)


def check_fixed_dequant_reduce(lib):
    """Eq. 8 with the global scale: every partial sum is an integer over s, hence exact, and
    the result is (sum q) / s times fl(1/N) with one rounding."""
    rng = np.random.default_rng(61)
    for bits, log2_s in ((4, 19), (8, 17)):
        n = 2001
        cb = oracle.code_bytes(n, bits)
        stride = cb + 7
        for W in (1, 2, 3, 8, 16, 17):
            codes = rng.integers(0, 256, W * stride, dtype=np.uint8)
            out = oracle.fixed_dequant_reduce(codes, W, n, bits, log2_s, code_stride_bytes=stride, lib=lib)
            tot = np.zeros(n)
            for w in range(W):
                tot += unpack(codes[w * stride:w * stride + cb], n, bits)
            d_sum = (tot * 2.0 ** -log2_s).astype(np.float32)          # exact: |sum q| < 2^24
            assert np.array_equal(out, d_sum * (np.float32(1.0) / np.float32(W)))
            ref = tot * 2.0 ** -log2_s / W
            if W in (1, 2, 8, 16):                                      # 1/W exact too
                assert np.array_equal(out, ref.astype(np.float32))
            else:
                assert np.all(np.abs(out - ref) <= np.abs(ref) * 2.0 ** -22)
        assert np.abs(tot).max() > 0


def check_fixed_edges(lib):
    """bf16 widening, empty input, odd length (last high nibble 0), threads agree, the state
    saturates at +-127/-128 instead of wrapping."""
    rng = np.random.default_rng(67)
    assert fcq(lib, np.zeros(0, np.float32), np.zeros(0, np.int8), 4, 19, 4, 0.25).size == 0
    n = 777
    s = 2.0 ** 19
    gb = to_bf16_bits((rng.standard_normal(n) * 4 / s).astype(np.float32))
    e0 = rng.integers(-128, 128, n).astype(np.int8)
    ea, eb, ec = e0.copy(), e0.copy(), e0.copy()
    ca = fcq(lib, gb, ea, 4, 19, 6, 0.25)
    cb = fcq(lib, bf16_bits_to_f32(gb), eb, 4, 19, 6, 0.25)
    cc = fcq(lib, gb, ec, 4, 19, 6, 0.25, threads=4)
    assert np.array_equal(ca, cb) and np.array_equal(ea, eb) and np.array_equal(ca, cc) and np.array_equal(ea, ec)
    assert ca.size == (n + 1) // 2 and (ca[-1] >> 4) == 0
    big = np.full(8, 1.0, np.float32)
    big[4:] = -1.0
    e8 = np.zeros(8, np.int8)
    c = fcq(lib, big, e8, 4, 19, 4, 1.0)
    assert unpack(c, 8, 4).tolist() == [7] * 4 + [-8] * 4 and e8.tolist() == [127] * 4 + [-128] * 4
    o1 = oracle.fixed_dequant_reduce(np.tile(ca, 3), 3, n, 4, 19, lib=lib)
    o4 = oracle.fixed_dequant_reduce(np.tile(ca, 3), 3, n, 4, 19, threads=4, lib=lib)
    assert np.array_equal(o1, o4)


def fcq32(lib, g, e, bits, log2_s, beta, reset=0):
    return oracle.fixed_compensate_quantize_f32state(g, e, bits, log2_s, beta, reset, lib=lib)


def check_fixed_f32state(lib):
    """The global scale of Eq. 1 with the compensation error kept in high precision (Table 9, the
    row without error compression): Alg. 1 with the 8-bit round trip of the state taken out."""
    # hand-worked dyadic example (Eq. 1-5): every code byte and state value
    rows = {}
    with open(os.path.join(GOLDEN, "worked_example_fixed_scale_f32_state_p4.txt")) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                key, *vals = line.split()
                rows[key] = vals
    bits, log2_s, beta = int(rows["bits"][0]), int(rows["log2_s"][0]), float(rows["beta"][0])
    g = np.array([float(v) for v in rows["g"]], np.float32)
    e = np.zeros(g.size, np.float32)
    for step in (0, 1):
        codes = fcq32(lib, g, e, bits, log2_s, beta)
        assert np.array_equal(codes, np.array([int(b, 16) for b in rows[f"bytes{step}"]], np.uint8)), (step, codes)
        assert unpack(codes, g.size, bits).tolist() == [int(v) for v in rows[f"q{step}"]]
        assert e.tolist() == [float(v) for v in rows[f"e{step + 1}"]], (step, e)

    rng = np.random.default_rng(71)
    for trial in range(200):
        bits = (4, 8)[trial & 1]
        qmin, qmax = qrange(bits)
        log2_s = int(rng.choice([19, 17, 10, 3, -2]))
        beta = float(rng.choice([0.25, 0.5, 1.0, 0.3, 0.9, 0.0]))
        s = 2.0 ** log2_s
        n = int(rng.integers(1, 300))
        g = (rng.standard_normal(n) * rng.choice([0.3, 1, 3, 30]) * qmax / s).astype(np.float32)
        e0 = (rng.standard_normal(n) * 0.4 / s).astype(np.float32) if trial % 3 else np.zeros(n, np.float32)
        e = e0.copy()
        codes = fcq32(lib, g, e, bits, log2_s, beta)
        q = unpack(codes, n, bits)
        h = g.astype(np.float64) + e0                                   # Eq. 2
        h32 = (g + e0).astype(np.float64)                               # the binary32 sum the oracle forms
        x = h32 * s                                                     # exact: s is a power of two
        want_q = np.clip(np.rint(x), qmin, qmax)                        # Eq. 1: nearest level, ties to even
        assert np.array_equal(q, want_q), (trial, x[q != want_q], q[q != want_q])
        assert np.all(np.abs(h32 - h) <= np.abs(h) * 2.0 ** -24 + 1e-300)
        unsat = np.abs(x) <= qmax + 0.5
        assert np.all(np.abs(h32 - q / s)[unsat] <= 0.5 / s)            # Lemma 5: |h - d| <= 1/(2s)
        b32 = np.float64(np.float32(beta))
        omb = np.float64(np.float32(1.0) - np.float32(beta))
        want_e = omb * e0 + b32 * (h32 - q / s)                         # Eq. 5 in binary64
        assert np.all(np.abs(e - want_e) <= np.abs(want_e) * 2.0 ** -23 + np.abs(b32 * (h32 - q / s)) * 2.0 ** -23 + 1e-45)
        if beta == 0.0:
            assert np.array_equal(e, e0)                                # the state never moves
        if beta == 1.0:
            assert np.array_equal(e.astype(np.float64), h32 - q / s)    # classic error feedback, Eq. 4 (exact)
        e_r = e0.copy()
        codes_r = fcq32(lib, g, e_r, bits, log2_s, beta, reset=1)       # Eq. 7: same payload, state 0
        assert np.array_equal(codes_r, codes) and not e_r.any()

    # Lemma 1 with an uncompressed state: sum d = sum g - e~_K / beta, up to binary32 rounding
    for bits, log2_s, beta, K in ((4, 19, 0.5, 12), (4, 17, 0.25, 20), (8, 19, 1.0, 8)):
        qmin, qmax = qrange(bits)
        s = 2.0 ** log2_s
        n = 4000
        e = np.zeros(n, np.float32)
        sum_d, sum_g = np.zeros(n), np.zeros(n)
        for _ in range(K):
            g = (rng.uniform(-(qmax - 1), qmax - 1, n) / s).astype(np.float32)          # never clamps
            codes = fcq32(lib, g, e, bits, log2_s, beta)
            sum_d += unpack(codes, n, bits) / s
            sum_g += g
        assert np.abs(e).max() > 0
        assert np.abs(sum_d - (sum_g - e.astype(np.float64) / beta)).max() <= 8 * K * 2.0 ** -24 * qmax / s / beta
        assert np.abs(sum_d - sum_g).max() <= 0.5 / s / beta * (1 + 1e-6)                # and it never accumulates

    # one step from a zero state is one step of the block-scaled form whose blocks all peak at qmax/s,
    # and of the 8-bit-state form wherever s_e e~' is an integer in range
    for bits, log2_s, B in ((4, 19, 256), (8, 17, 64)):
        qmin, qmax = qrange(bits)
        s = 2.0 ** log2_s
        n = 20 * B
        g = (rng.uniform(-qmax, qmax, n) / s).astype(np.float32)
        g[np.arange(0, n, B) + rng.integers(0, B, n // B)] = np.float32(qmax / s)
        e_f, e_b = np.zeros(n, np.float32), np.zeros(n, np.float32)
        c_f = fcq32(lib, g, e_f, bits, log2_s, 0.25)
        c_b, _ = cq(lib, g, e_b, bits, B, 0.25)
        assert np.array_equal(c_f, c_b) and np.array_equal(e_f, e_b)
    m = rng.integers(-40, 41, 2000)                                     # g = m/16 with s = 8: h*s on half integers
    g = (m / 16.0).astype(np.float32)
    e32, e8 = np.zeros(g.size, np.float32), np.zeros(g.size, np.int8)
    c32 = fcq32(lib, g, e32, 4, 3, 0.5)
    c8 = fcq(lib, g, e8, 4, 3, 4, 0.5)
    fits = np.abs(e32 * 32) <= 127
    assert np.array_equal(c32, c8) and np.array_equal((e32 * 32)[fits], e8[fits].astype(np.float32)) and fits.mean() > 0.5

    # edges: empty, odd length, bf16 widening, clamp on huge values
    assert fcq32(lib, np.zeros(0, np.float32), np.zeros(0, np.float32), 4, 19, 0.25).size == 0
    n = 777
    gb = to_bf16_bits((rng.standard_normal(n) * 4 / 2.0 ** 19).astype(np.float32))
    ea, eb = np.zeros(n, np.float32), np.zeros(n, np.float32)
    ca, cb_ = fcq32(lib, gb, ea, 4, 19, 0.25), fcq32(lib, bf16_bits_to_f32(gb), eb, 4, 19, 0.25)
    assert np.array_equal(ca, cb_) and np.array_equal(ea, eb) and ca.size == (n + 1) // 2 and (ca[-1] >> 4) == 0
    big = np.array([3e38, -3e38, 1.0, -1.0], np.float32)
    e = np.zeros(4, np.float32)
    assert unpack(fcq32(lib, big, e, 4, 19, 1.0), 4, 4).tolist() == [7, -8, 7, -8]
    assert e[2] == np.float32(1.0 - 7 / 2.0 ** 19) and e[3] == np.float32(-1.0 + 8 / 2.0 ** 19)


def check_clip(lib):
    """Clipping to [-c, c]: values inside are untouched, values outside land on +-c with their
    sign, c = inf is the identity, the map is idempotent, and bf16 input is widened first."""
    rng = np.random.default_rng(71)
    g = rng_grad(rng, 5000, "student", 1e-3)
    g[:4] = [0.0, -0.0, 1e30, -1e30]
    for c in (np.float32(1e-3), np.float32(3.3e-4), np.float32(2.0 ** -12)):
        out = oracle.clip_gradient(g, c, lib=lib)
        inside = np.abs(g) <= c
        assert inside.any() and (~inside).any()
        assert np.array_equal(out[inside], g[inside])
        assert np.all(out[~inside] == np.sign(g[~inside]) * c)
        assert np.array_equal(oracle.clip_gradient(out, c, lib=lib), out)
    assert np.array_equal(oracle.clip_gradient(g, np.inf, lib=lib), g)
    gb = to_bf16_bits(g)
    c = np.float32(7.7e-4)                              # not a bf16 value
    out = oracle.clip_gradient(gb, c, lib=lib)
    assert np.array_equal(out, np.clip(bf16_bits_to_f32(gb), -c, c)) and (out == c).any()


def check_optimizer_steps(lib):
    """Eq. 9 and Eq. 10 as written (no bias correction, delta inside the root, m_0 = v_0 = 0):
    closed forms for a constant gradient, the unrolled recurrences in binary64 for a varying
    one, beta1 = 1 (no momentum), a zero gradient, and the sign symmetry of the update."""
    rng = np.random.default_rng(83)
    n, K = 2000, 9
    eta, b1, b2, dl = 1e-3, 0.1, 0.02, 1e-8
    # SGD: theta_K = theta_0 - eta * sum g
    th0 = rng.standard_normal(n).astype(np.float32)
    th = th0.copy()
    gs = [rng_grad(rng, n, "normal", 1e-2) for _ in range(K)]
    for g in gs:
        oracle.sgd_update(th, g, eta, lib=lib)
    want = th0 - eta * np.sum(np.stack(gs).astype(np.float64), axis=0)
    assert np.abs(th - want).max() <= K * 2.0 ** -23 * np.abs(th0).max()
    assert np.abs(th - th0).max() > 1e-5
    # Adam family, varying gradient: unrolled in binary64
    th = th0.copy()
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    m64, v64, th64 = np.zeros(n), np.zeros(n), th0.astype(np.float64)
    f = lambda x: np.float64(np.float32(x))
    for g in gs:
        oracle.adam_update(th, m, v, g, eta, b1, b2, dl, lib=lib)
        m64 = (1 - f(b1)) * m64 + f(b1) * g
        v64 = (1 - f(b2)) * v64 + f(b2) * g.astype(np.float64) ** 2
        th64 = th64 - f(eta) / np.sqrt(v64 + f(dl)) * m64
    assert np.abs(m - m64).max() <= K * 2.0 ** -22 * np.abs(m64).max()
    assert np.abs(v - v64).max() <= K * 2.0 ** -22 * np.abs(v64).max()
    assert np.abs(th - th64).max() <= K * 2.0 ** -21 * np.abs(th0).max()
    assert np.abs(th - th0).max() > 1e-3                       # steps of order eta/sqrt(beta2) each
    # constant gradient c: m_k = c (1 - (1-b1)^k), v_k = c^2 (1 - (1-b2)^k)
    c = np.float32(3e-3)
    th = np.zeros(4, np.float32)
    m, v = np.zeros(4, np.float32), np.zeros(4, np.float32)
    g = np.full(4, c, np.float32)
    for k in range(1, 6):
        oracle.adam_update(th, m, v, g, eta, b1, b2, 0.0, lib=lib)
        assert abs(m[0] / (c * (1 - (1 - f(b1)) ** k)) - 1) < 1e-6
        assert abs(v[0] / (f(c) ** 2 * (1 - (1 - f(b2)) ** k)) - 1) < 1e-6
    # first step from zero moments, delta = 0: theta_1 = -eta * b1 * g / (sqrt(b2) |g|) whatever |g|
    for scale in (1e-6, 1.0, 1e4):
        th = np.zeros(2, np.float32)
        m, v = np.zeros(2, np.float32), np.zeros(2, np.float32)
        oracle.adam_update(th, m, v, np.array([scale, -scale], np.float32), eta, b1, b2, 0.0, lib=lib)
        step = f(eta) * f(b1) / np.sqrt(f(b2))
        assert abs(th[0] / -step - 1) < 1e-6 and th[1] == -th[0]
    # beta1 = 1: no momentum; zero gradient: moments decay, theta moves only by the old momentum
    th = th0.copy()
    m, v = rng_grad(rng, n, "normal", 1e-2), np.abs(rng_grad(rng, n, "normal", 1e-4))
    g = rng_grad(rng, n, "normal", 1e-2)
    oracle.adam_update(th, m, v, g, eta, 1.0, b2, dl, lib=lib)
    assert np.array_equal(m, g)
    m0, v0, th1 = m.copy(), v.copy(), th.copy()
    oracle.adam_update(th, m, v, np.zeros(n, np.float32), eta, b1, b2, dl, lib=lib)
    assert np.allclose(m, (1 - f(b1)) * m0, rtol=1e-6) and np.allclose(v, (1 - f(b2)) * v0, rtol=1e-6)
    assert np.all(np.sign(th1 - th) == np.sign(m))


def check_round_to_bf16(lib):
    """fp32 -> bf16, ties to even: the result is one of the two neighbouring bf16 values, the
    nearer one, the even one at an exact tie; bf16 inputs come back unchanged; and the whole
    map agrees with torch's own conversion on every exponent and on random bits."""
    import torch
    rng = np.random.default_rng(89)
    bits = np.concatenate([rng.integers(0, 2 ** 32, 200000, dtype=np.uint64).astype(np.uint32),
                           (np.arange(0, 256, dtype=np.uint32) << 23) | 0x00008000,      # exact ties, even below
                           (np.arange(0, 256, dtype=np.uint32) << 23) | 0x00018000,      # exact ties, odd below
                           (np.arange(0, 256, dtype=np.uint32) << 23) | 0x00007FFF,
                           (np.arange(0, 256, dtype=np.uint32) << 23) | 0x00008001,
                           np.array([0, 0x80000000, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F800000, 0x00000001], np.uint32)])
    x = bits.view(np.float32)
    x = x[np.isfinite(x) | np.isinf(x)]
    got = oracle.round_to_bf16(x, lib=lib)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    back = bf16_bits_to_f32(got).astype(np.float64)
    fin = np.isfinite(back) & np.isfinite(x)
    lo = bf16_bits_to_f32((x.view(np.uint32) >> 16).astype(np.uint16)).astype(np.float64)   # truncation
    assert np.all(np.abs(back[fin] - x[fin]) <= np.abs(x[fin] - lo[fin]) + 0.0)              # never worse than truncating
    tie = (x.view(np.uint32) & 0xFFFF) == 0x8000
    assert np.all((got[tie & fin] & 1) == 0)                                                  # ties land on even
    exact = (x.view(np.uint32) & 0xFFFF) == 0
    assert np.array_equal(got[exact], (x.view(np.uint32)[exact] >> 16).astype(np.uint16))
    assert np.all(np.isnan(bf16_bits_to_f32(oracle.round_to_bf16(np.array([np.nan, -np.nan], np.float32), lib=lib))))


def check_bf16_scales(lib):
    """Block steps kept in bf16: the stored step is the binary32 step max|h|/qmax rounded to
    the nearest bf16 (checked against torch's conversion), and everything else follows Eq. 1-5
    with that rounded step: nearest level by brute force, the rounding bound of Lemma 5,
    d + delta = h with d decoded by the receiver from the bf16 step, the telescoping identity
    of Lemma 1, and Eq. 8 equal to the binary32-step reduce fed the widened steps."""
    import torch
    as_bf16 = lambda x: torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16) \
        .view(torch.int16).numpy().view(np.uint16)
    # the dyadic worked example has a step that bf16 holds exactly: same bytes, same state
    g = (np.array([7, -3.5, 2.5, 0.5, 1.5, -0.25, 0, -7]) * 2.0 ** -10).astype(np.float32)
    e = np.zeros(8, np.float32)
    codes, s16 = oracle.compensate_quantize(g, e, 4, 8, 0.25, bf16_scales=True, lib=lib)
    assert codes.tolist() == [0xC7, 0x02, 0x02, 0x90] and s16.tolist() == [0x3A80]
    assert np.array_equal(e * 2.0 ** 10, [0, .125, .125, .125, -.125, -.0625, 0, 0])

    rng = np.random.default_rng(97)
    for bits, B, kind in ((4, 256, "student"), (8, 64, "normal"), (4, 32, "wide"), (8, 512, "student")):
        qmin, qmax = qrange(bits)
        n = 50 * B + 9
        g = rng_grad(rng, n, kind)
        e0 = rng_grad(rng, n, "normal", 1e-4)
        h = g + e0
        e = e0.copy()
        codes, s16 = oracle.compensate_quantize(g, e, bits, B, 1.0, bf16_scales=True, lib=lib)
        assert s16.dtype == np.uint16
        nb = oracle.num_blocks(n, B)
        amax = np.array([np.abs(h[b * B:min(n, (b + 1) * B)]).max() for b in range(nb)], np.float32)
        want = as_bf16(amax / np.float32(qmax))
        assert np.array_equal(s16, want)
        assert (s16 & 0x7F).any()                           # steps that are not powers of two
        assert np.any(s16 != (((amax / np.float32(qmax)).view(np.uint32)) >> 16))  # some rounded up
        D = bf16_bits_to_f32(s16)[block_index(n, B)].astype(np.float64)
        q = unpack(codes, n, bits)
        x = h.astype(np.float64) / D
        assert np.all(np.abs(q - x) <= 0.5 + 4 * qmax * 2.0 ** -24)        # nearest level, Lemma 5
        assert q.min() >= -qmax and q.max() <= qmax
        assert np.all(np.abs(e) <= D * (0.5 + 4 * qmax * 2.0 ** -24))
        top = np.array([b * B + np.argmax(np.abs(h[b * B:min(n, (b + 1) * B)])) for b in range(nb)])
        assert np.all(np.abs(q[top]) == qmax)
        # receiver's decode from the bf16 steps + the sender's error gives back h (Eq. 4)
        d = oracle.dequant_reduce(codes, s16, 1, n, bits, B, lib=lib)
        with np.errstate(divide="ignore", invalid="ignore"):
            ratio = np.where(d != 0, h.astype(np.float64) / d.astype(np.float64), 1.0)
        safe = (d == 0) | ((ratio >= 0.5) & (ratio <= 2.0))
        assert safe.mean() > 0.99
        assert np.array_equal((d + e).astype(np.float32)[safe], h[safe])
        assert np.array_equal(d, (q * D).astype(np.float32))

    # Eq. 8: the bf16-step reduce is the binary32-step reduce of the widened steps
    bits, B, W, n = 4, 64, 5, 64 * 33 + 3
    payload_c, payload_s = [], []
    for w in range(W):
        gw = rng_grad(rng, n, "student")
        cw, sw = oracle.compensate_quantize(gw, np.zeros(n, np.float32), bits, B, 0.25, bf16_scales=True, lib=lib)
        payload_c.append(cw); payload_s.append(sw)
    C, S = np.concatenate(payload_c), np.concatenate(payload_s)
    a = oracle.dequant_reduce(C, S, W, n, bits, B, lib=lib)
    b = oracle.dequant_reduce(C, bf16_bits_to_f32(S), W, n, bits, B, lib=lib)
    assert np.array_equal(a, b) and np.any(a != 0)
    assert np.array_equal(a, oracle.dequant_reduce(C, S, W, n, bits, B, threads=3, lib=lib))

    # Lemma 1 (same decompressor on both sides): sum_k d_k = sum_k g_k - e~_K / beta
    bits, B, beta, K, n = 4, 128, 0.25, 12, 128 * 20
    e = np.zeros(n, np.float32)
    sum_d, sum_g = np.zeros(n), np.zeros(n)
    for k in range(K):
        gk = rng_grad(rng, n, "normal")
        ck, sk = oracle.compensate_quantize(gk, e, bits, B, beta, bf16_scales=True, lib=lib)
        sum_d += oracle.dequant_reduce(ck, sk, 1, n, bits, B, lib=lib)
        sum_g += gk
    gap = np.abs(sum_d - (sum_g - e.astype(np.float64) / beta))
    assert gap.max() <= 20 * K * 2.0 ** -24 * 1e-3 * 8 and np.abs(e).max() > 0

    # zero and subnormal steps: the test is made on the rounded step
    tiny = np.float32(FLT_MIN)
    g = np.zeros(24, np.float32)
    g[0] = np.float32(7) * tiny * np.float32(1 - 2.0 ** -10)   # step just under FLT_MIN, rounds up to it
    g[8] = np.float32(7) * tiny * np.float32(0.25)             # subnormal step also after rounding
    e = np.zeros(24, np.float32)
    codes, s16 = oracle.compensate_quantize(g, e, 4, 8, 1.0, bf16_scales=True, lib=lib)
    assert s16.tolist() == [0x0080, 0, 0]
    q = unpack(codes, 24, 4)
    assert q[0] == 7 and not q[1:].any()
    assert e[8] == g[8] and e[0] == g[0] - np.float32(7) * tiny
    # threads and odd sizes
    g = rng_grad(rng, 1003, "student")
    e1, e2 = np.zeros(1003, np.float32), np.zeros(1003, np.float32)
    r1 = oracle.compensate_quantize(g, e1, 8, 32, 0.5, bf16_scales=True, lib=lib)
    r2 = oracle.compensate_quantize(g, e2, 8, 32, 0.5, bf16_scales=True, threads=4, lib=lib)
    assert np.array_equal(r1[0], r2[0]) and np.array_equal(r1[1], r2[1]) and np.array_equal(e1, e2)


FIXED_CHECKS = [
    check_bf16_scales,
    check_round_to_bf16,
    check_clip,
    check_optimizer_steps,
    check_fixed_worked_example,
    check_fixed_nearest_levels,
    check_fixed_zero_error_fixed_point,
    check_fixed_telescoping,
    check_fixed_beta_and_reset,
    check_fixed_matches_block_form,
    check_fixed_dequant_reduce,
    check_fixed_edges,
    check_fixed_f32state,
]
ALL_CHECKS = ALL_CHECKS + FIXED_CHECKS
