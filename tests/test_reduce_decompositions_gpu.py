"""Every work decomposition of the reduce (Alg. 1 step 3 / Eq. 8) against the oracle: the
quad layout with scalar or lane-loaded block steps, and the wide code loads with the LDS
transpose, over worker counts on both sides of the library's own switch points, ragged
lengths, arbitrary code values (including the clamp code) and steps too large for the
16 D shortcut.  All must give the oracle's averaged gradient bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_dequant_reduce, loco_dequant_reduce_decomposed,
                                  loco_dequant_reduce_decomposition, loco_num_blocks)
from paper_2407_04480_amd.binding import LocoError

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
QUAD, QUAD_LANE_STEPS, WIDE4, WIDE8, WIDE16 = 1, 2, 3, 4, 5


def exists(decomposition, bits, B):
    if decomposition == QUAD_LANE_STEPS:
        return B >= 128
    if decomposition == WIDE4:
        return bits == 4
    return True


def random_payloads(rs, W, n, bits, B, code_pad=0, scale_pad=0, huge=False):
    cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B)
    cs, ss = (cb + 15) // 16 * 16 + 16 * code_pad, nb + scale_pad
    codes = rs.integers(0, 256, W * cs, dtype=np.uint8)
    scales = (rs.uniform(0.5, 2.0, W * ss) * np.exp2(rs.integers(-30, -5, W * ss))).astype(np.float32)
    scales[rs.integers(0, W * ss, max(1, W * ss // 50))] = 0.0            # dead blocks
    if huge:
        scales[rs.integers(0, W * ss, max(1, W * ss // 40))] = np.float32(2.0 ** 120)   # 16 D is not taken from here up
    return codes, scales, cs, ss


@pytest.mark.parametrize("decomposition", [QUAD, QUAD_LANE_STEPS, WIDE4, WIDE8, WIDE16])
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("B", [32, 64, 128, 256, 512])
def test_every_decomposition_matches_the_oracle(decomposition, bits, B):
    rs = np.random.default_rng(1000 * decomposition + 10 * B + bits)
    cases = [(1, 1), (2, 7), (3, 4097), (5, 2048 * 9), (4, 100_003), (9, 33 * 1024 + 517), (13, 2048 * 21 + 3),
             (27, 2048 * 5 + 77)]
    for W, n in cases:
        # W = 5, 13, 27: a few steps of 2^120, for which 4-bit tiles are summed again without the shortcut
        # (one chunk and a rest; three chunks and a rest, which is the pipelined loop; six and a rest)
        codes, scales, cs, ss = random_payloads(rs, W, n, bits, B, code_pad=W % 3, scale_pad=W % 2,
                                                huge=(W in (5, 13, 27) and bits == 4))
        out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
        args = (torch.from_numpy(codes).to(DEV), cs, torch.from_numpy(scales).to(DEV), ss, W, n, bits, B, out)
        if not exists(decomposition, bits, B):
            with pytest.raises(LocoError) as ei:
                loco_dequant_reduce_decomposed(*args, decomposition)
            assert ei.value.status == 2
            return
        loco_dequant_reduce_decomposed(*args, decomposition)
        torch.cuda.synchronize()
        want = oracle.dequant_reduce(codes, scales, W, n, bits, B, cs, ss)
        got = out.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)) or np.array_equal(got, want), \
            f"decomposition {decomposition} bits={bits} B={B} W={W} n={n}: {np.count_nonzero(got != want)} differ"


@pytest.mark.parametrize("bits,B,W", [(4, 32, 7), (4, 64, 8), (4, 32, 15), (4, 32, 16), (4, 64, 33), (4, 64, 63), (4, 64, 64), (4, 128, 70),
                                      (4, 256, 63), (4, 256, 64), (4, 256, 130), (4, 512, 128), (8, 64, 40),
                                      (8, 64, 95), (8, 64, 96), (8, 256, 1), (8, 256, 2), (8, 512, 9), (8, 512, 100)])
def test_the_librarys_own_choice_matches_the_oracle(bits, B, W):
    """loco_dequant_reduce itself on both sides of every switch point of its dispatch."""
    rs = np.random.default_rng(7 * W + B + bits)
    n = 3 * 8192 + 1111
    codes, scales, cs, ss = random_payloads(rs, W, n, bits, B)
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    loco_dequant_reduce(torch.from_numpy(codes).to(DEV), cs, torch.from_numpy(scales).to(DEV), ss, W, n, bits, B, out)
    torch.cuda.synchronize()
    want = oracle.dequant_reduce(codes, scales, W, n, bits, B, cs, ss)
    assert np.array_equal(out.cpu().numpy(), want), f"bits={bits} B={B} W={W}"
    chosen = loco_dequant_reduce_decomposition(W, bits, B)
    assert 1 <= chosen <= 5 and exists(chosen, bits, B)


def test_large_shard_with_many_payloads_through_the_librarys_choice():
    """From 2^22 elements on 64 payloads of 4-bit codes take the 16-byte code loads; below, the quad layout."""
    rs = np.random.default_rng(5)
    bits, B, W = 4, 256, 64
    for n in ((1 << 22) + 2048 * 3 + 5, (1 << 22) - 2048 - 1):
        codes, scales, cs, ss = random_payloads(rs, W, n, bits, B)
        out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
        loco_dequant_reduce(torch.from_numpy(codes).to(DEV), cs, torch.from_numpy(scales).to(DEV), ss, W, n, bits, B, out)
        torch.cuda.synchronize()
        want = oracle.dequant_reduce(codes, scales, W, n, bits, B, cs, ss, threads=8)
        assert np.array_equal(out.cpu().numpy(), want), f"n={n}"


def test_many_workers_take_the_wide_loads():
    assert loco_dequant_reduce_decomposition(8, 4, 256) == QUAD
    assert loco_dequant_reduce_decomposition(16, 4, 256) == QUAD
    assert loco_dequant_reduce_decomposition(64, 4, 256) == WIDE16
    assert loco_dequant_reduce_decomposition(128, 4, 256) == WIDE16
    assert loco_dequant_reduce_decomposition(7, 4, 64) == QUAD
    assert loco_dequant_reduce_decomposition(8, 4, 64) == WIDE4
    assert loco_dequant_reduce_decomposition(8, 4, 128) == QUAD
    assert loco_dequant_reduce_decomposition(16, 4, 64) == WIDE8
    assert loco_dequant_reduce_decomposition(64, 4, 64) == WIDE16
    assert loco_dequant_reduce_decomposition(8, 8, 64) == QUAD
    assert loco_dequant_reduce_decomposition(64, 8, 64) == QUAD
    assert loco_dequant_reduce_decomposition(128, 8, 64) == WIDE16
    assert loco_dequant_reduce_decomposition(8, 8, 256) == QUAD_LANE_STEPS
    assert loco_dequant_reduce_decomposition(8, 3, 64) == -1 and loco_dequant_reduce_decomposition(0, 4, 64) == -1
