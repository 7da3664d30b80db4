"""The reduce when the payloads are many and large (8 or more payloads holding 2^33 bytes of
codes or more), where the library hands the tiles to the XCDs in the hardware's own order instead
of runs of 32.  Alg. 1 step 3 / Eq. 8 does not care: the result must be the same bits as with the
other order, which the library takes when the payload strides are multiples of 4 KiB, and the same
bits as the oracle's on slices of the array (head, a middle piece, the ragged tail)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_04480_amd import (loco_code_bytes, loco_dequant_reduce, loco_dequant_reduce_fixed, loco_num_blocks)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def round_up(x, m):
    return (x + m - 1) // m * m


def payload_slices(codes, scales, W, cs, ss, lo, hi, bits, B):
    """Host copies of elements [lo, hi) of every payload, packed back to back; lo is a multiple of 4096."""
    cb_lo, cb_hi = lo * bits // 8, (hi * bits + 7) // 8
    sb_lo, sb_hi = lo // B, (hi + B - 1) // B
    c = torch.cat([codes[w * cs + cb_lo:w * cs + cb_hi] for w in range(W)]).cpu().numpy()
    s = None if scales is None else torch.cat([scales[w * ss + sb_lo:w * ss + sb_hi] for w in range(W)]).cpu().numpy()
    return c, s, cb_hi - cb_lo, sb_hi - sb_lo


# (form, bits, B, W, n): quad 8-bit, quad with lane-loaded steps, 8-byte code loads, quad 4-bit, fixed-scale
CASES = [("block", 8, 64, 16, 842301952 - 3), ("block", 8, 256, 16, 842301952 - 3), ("block", 4, 64, 32, 842301952 - 3),
         ("block", 4, 128, 12, 1500000000 - 5), ("fixed", 4, 0, 24, 842301952 - 3)]


@pytest.mark.parametrize("form,bits,B,W,n", CASES)
def test_both_tile_orders_give_the_oracles_bits(form, bits, B, W, n):
    gen = torch.Generator(device=DEV).manual_seed(17 * W + bits)
    cb = loco_code_bytes(n, bits)
    nb = loco_num_blocks(n, B) if form == "block" else 0
    cs1, ss1 = round_up(cb, 16) + 48, nb + 5                 # not multiples of 4 KiB: the hardware's own order
    cs2, ss2 = round_up(cb, 4096), round_up(nb, 1024)        # multiples of 4 KiB: runs of tiles per XCD
    assert W >= 8 and W * cb >= 2 ** 33 and cs1 % 4096 != 0 and (form == "fixed" or (ss1 * 4) % 4096 != 0)
    print(f"[large span] {form} bits={bits} B={B} W={W} n={n}: {W * cb / 2**30:.1f} GiB of codes", flush=True)
    codes1 = torch.randint(0, 256, (W * cs1,), dtype=torch.uint8, device=DEV, generator=gen)
    codes2 = torch.zeros(W * cs2, dtype=torch.uint8, device=DEV)
    for w in range(W):
        codes2[w * cs2:w * cs2 + cb] = codes1[w * cs1:w * cs1 + cb]
    scales1 = scales2 = None
    if form == "block":
        scales1 = (torch.rand(W * ss1, device=DEV, generator=gen) + 0.5) * 1e-4
        scales1[torch.randint(0, W * ss1, (W * ss1 // 64,), device=DEV, generator=gen)] = 0.0     # dead blocks
        scales2 = torch.zeros(W * ss2, dtype=torch.float32, device=DEV)
        for w in range(W):
            scales2[w * ss2:w * ss2 + nb] = scales1[w * ss1:w * ss1 + nb]
    out1 = torch.full((n,), 7.0, dtype=torch.float32, device=DEV)
    out2 = torch.full((n,), 9.0, dtype=torch.float32, device=DEV)
    if form == "block":
        loco_dequant_reduce(codes1, cs1, scales1, ss1, W, n, bits, B, out1)
        loco_dequant_reduce(codes2, cs2, scales2, ss2, W, n, bits, B, out2)
    else:
        loco_dequant_reduce_fixed(codes1, cs1, W, n, bits, 19, out1)
        loco_dequant_reduce_fixed(codes2, cs2, W, n, bits, 19, out2)
    torch.cuda.synchronize()
    assert torch.equal(out1.view(torch.int32), out2.view(torch.int32)), "the two tile orders disagree"
    del codes2, scales2, out2
    for lo, hi in ((0, 3 * 4096 + 77), (n // 2 // 4096 * 4096, n // 2 // 4096 * 4096 + 8192), ((n - 9000) // 4096 * 4096, n)):
        c, s, ccs, sss = payload_slices(codes1, scales1, W, cs1, ss1, lo, hi, bits, max(B, 1))
        if form == "block":
            want = oracle.dequant_reduce(c, s, W, hi - lo, bits, B, ccs, sss)
        else:
            want = oracle.fixed_dequant_reduce(c, W, hi - lo, bits, 19, ccs)
        got = out1[lo:hi].cpu().numpy()
        assert np.array_equal(got, want), f"elements [{lo}, {hi}): {np.count_nonzero(got != want)} differ"
