"""Host-side bounds model of the two attention kernels that take grids their block side does not
divide (short edge blocks filled with clamped copies).  It mirrors the kernels' address arithmetic
- direct global -> LDS transfers add an UNSIGNED 32-bit lane offset to a scalar base, ordinary
loads and stores use signed offsets - and checks that every address stays inside the (batch, head)
slice.  A lane offset that underflows wraps to +4 GiB: that is the fault this test guards against."""
import pytest

M32 = 1 << 32
def u32(x): return x % M32
def s32(x):
    x %= M32
    return x - M32 if x >= (1 << 31) else x

def check_block16(gh, gw, bm=1):
    rowB = 128; gridrowB = gw * rowB; T = 1 + gh * gw; size = T * rowB
    nbh, nbw = (gh + 15) // 16, (gw + 15) // 16
    hv_last, wv_last = gh - 16 * (nbh - 1), gw - 16 * (nbw - 1)
    rows_of = lambda Rb: hv_last if Rb == nbh - 1 else 16
    cols_of = lambda Cb: wv_last if Cb == nbw - 1 else 16
    tile_token = lambda Rb, Cb, sub: 1 + (Rb * 16 + sub * 4) * gw + Cb * 16
    def tile_off(i, sub, hv, wv):
        r = min(4 * sub + (i >> 4), hv - 1) - 4 * sub
        return u32(u32(r * gw + min(i & 15, wv - 1)) * rowB)
    bad = 0
    for R in range(nbh):
        for C in range(nbw):
            for wave in range(4):
                for lane in range(64):
                    l32, hh, drow = lane & 31, lane >> 5, lane >> 3
                    # Q loads / O stores
                    for nt in range(2):
                        qoff = u32(tile_off(l32 + 32 * nt, wave, rows_of(R), cols_of(C)) + 64 * hh)
                        a = tile_token(R, C, wave) * rowB + s32(qoff)
                        if not (0 <= a and a + 64 <= size): bad += 1
                        i = l32 + 32 * nt
                        r = min(4 * wave + (i >> 4), rows_of(R) - 1) - 4 * wave
                        a = tile_token(R, C, wave) * rowB + (r * gw + min(i & 15, cols_of(C) - 1)) * rowB
                        if not (rowB <= a and a + 128 <= size): bad += 1
                    # transfers of every key tile of the neighbourhood
                    dma_koff = [drow * rowB + 16 * ((lane & 7) ^ ((drow >> 1) & 7)), drow * rowB + 16 * ((lane & 7) ^ ((4 + (drow >> 1)) & 7))]
                    RB, CB = R // bm, C // bm          # the block (bm x bm squares) this square lies in
                    R0, R1 = max(RB - 1, 0) * bm, min((RB + 2) * bm, nbh) - 1
                    C0, C1 = max(CB - 1, 0) * bm, min((CB + 2) * bm, nbw) - 1
                    if not (0 <= R0 <= R <= R1 < nbh and 0 <= C0 <= C <= C1 < nbw): bad += 1
                    for ir in range(R0, R1 + 1):
                        for ic in range(C0, C1 + 1):
                            for isub in range((hv_last + 3) // 4 if ir == nbh - 1 else 4):   # tiles with rows of their own
                                grow = min(4 * isub + wave, rows_of(ir) - 1)
                                base = u32(tile_token(ir, ic, 0) * rowB + grow * gridrowB)
                                for j in range(2):
                                    if ic == nbw - 1 and wv_last < 16:
                                        shift = u32((min(8 * j + drow, wv_last - 1) - drow) * rowB)
                                        a = base + u32(dma_koff[j] + shift)
                                    else:
                                        a = base + j * 8 * rowB + dma_koff[j]
                                    if not (rowB <= a and a + 16 <= size): bad += 1
                                    if bad > 5: return bad
    return bad

def check_sweep(gh, gw):
    rowB = 128; gridrowB = gw * rowB; T = 1 + gh * gw; size = T * rowB
    nbh, nbw = (gh + 7) // 8, (gw + 7) // 8
    hv_last, wv_last = gh - 8 * (nbh - 1), gw - 8 * (nbw - 1)
    bad = 0
    block_token = lambda Rb, Cb: 1 + Rb * 8 * gw + Cb * 8
    tile_off = lambda i, hv, wv: u32((min(i >> 3, hv - 1) * gw + min(i & 7, wv - 1)) * rowB)
    for R in range(nbh):
        hvq = hv_last if R == nbh - 1 else 8
        r0, r1 = max(R - 1, 0), min(R + 1, nbh - 1)
        for wave in range(4):
            for lane in range(64):
                l32, hh, drow = lane & 31, lane >> 5, lane >> 3
                dma_koff = [drow * rowB + 16 * ((lane & 7) ^ ((drow >> 1) & 7)), drow * rowB + 16 * ((lane & 7) ^ ((4 + (drow >> 1)) & 7))]
                for qc in range(nbw):
                    back = max((l32 & 7) - (wv_last - 1), 0) * rowB if (qc == nbw - 1 and wv_last < 8) else 0
                    for nt in range(2):
                        qoff = u32(tile_off(l32 + 32 * nt, hvq, 8) + 64 * hh)
                        a = block_token(R, qc) * rowB + u32(qoff - back)
                        if not (rowB <= a and a + 64 <= size): bad += 1
                        i = l32 + 32 * nt
                        wvq = wv_last if qc == nbw - 1 else 8
                        a = (block_token(R, qc) + min(i >> 3, hvq - 1) * gw + min(i & 7, wvq - 1)) * rowB
                        if not (rowB <= a and a + 128 <= size): bad += 1
                    # logits store (lane = key)
                    wvc = wv_last if qc == nbw - 1 else 8
                    kr, kc = min(lane >> 3, hvq - 1), min(lane & 7, wvc - 1)
                    tok = block_token(R, qc) + kr * gw + kc
                    if not (1 <= tok < T): bad += 1
                for ic in range(nbw):
                    for ir in range(r1 - r0 + 1):
                        hvk = hv_last if r0 + ir == nbh - 1 else 8
                        base = block_token(r0 + ir, ic) * rowB
                        back = max(drow - (wv_last - 1), 0) * rowB if (ic == nbw - 1 and wv_last < 8) else 0
                        for j in range(2):
                            a = base + min(2 * wave + j, hvk - 1) * gridrowB + u32(dma_koff[j] - back)
                            if not (rowB <= a and a + 16 <= size): bad += 1
                            if bad > 5: return bad
    return bad



@pytest.mark.parametrize("gh,gw", [(20, 27), (37, 21), (16, 50), (33, 16), (1, 1), (5, 70), (19, 30), (3, 3), (17, 17)])
def test_block16_kernel_addresses_stay_in_bounds(gh, gw):
    assert check_block16(gh, gw) == 0


@pytest.mark.parametrize("gh,gw,bm", [(37, 21, 2), (50, 70, 2), (70, 53, 4), (33, 16, 3), (5, 5, 4)])
def test_block16_kernel_addresses_with_larger_blocks(gh, gw, bm):
    assert check_block16(gh, gw, bm) == 0


@pytest.mark.parametrize("gh,gw", [(20, 27), (9, 9), (8, 100), (17, 8), (1, 1), (5, 5), (12, 30), (23, 33)])
def test_sweep_kernel_addresses_stay_in_bounds(gh, gw):
    assert check_sweep(gh, gw) == 0


def test_addresses_stay_in_bounds_on_random_grids():
    """A seeded sample of grid shapes (sides 1..75) through both address models, with blocks of one,
    two and four 16x16 squares for the block kernel."""
    import random
    rng = random.Random(2024)
    for _ in range(24):
        gh, gw = rng.randint(1, 75), rng.randint(1, 75)
        assert check_sweep(gh, gw) == 0, (gh, gw)
        assert check_block16(gh, gw, rng.choice([1, 2, 4])) == 0, (gh, gw)
