"""Host-side model of the global load addresses of the LDS-tiled stage-1 kernel
(csrc/fs_stage1_tiled2.hpp, fetch_w / fetch_h): every address a launch can form -- including the
prefetches that run past the end of K and the rows past V or B, whose values are never used --
must lie inside the W and H buffers.  The model restates the kernel's clamping arithmetic; it
exists to catch a clamp that forgets short rows (D < 64) or a short last tile."""
import itertools

import pytest

KS = 64


def w_addresses(D, V, VT, threads, WB=2):
    """Element offsets (in W elements) of every 16-byte W load of one launch."""
    WEPC = 16 // WB
    WCH = KS // WEPC
    WRPP = threads // WCH
    NWL = VT // WRPP
    nk = (D + KS - 1) // KS
    out = []
    for tile in range((V + VT - 1) // VT):
        tile_row0 = tile * VT
        for step in range(nk + 4):                      # steps past nk are the over-run prefetches
            k0 = step * KS
            over = k0 >= D
            for tid in range(threads):
                chunk, wrow = tid % WCH, tid // WCH
                k = chunk * WEPC if over else k0 + chunk * WEPC
                k = min(k, D - WEPC)
                for i in range(NWL):
                    row = min(tile_row0 + wrow + WRPP * i, V - 1)
                    row = tile_row0 if over else row
                    out.append((row * D + k, WEPC))
    return out


def h_addresses(D, B, BT, threads):
    RPP = threads // 8
    partial = BT < RPP
    hloads = 1 if partial else BT // RPP
    nk = (D + KS - 1) // KS
    out = []
    for bt in range((B + BT - 1) // BT):
        b0 = bt * BT
        for step in range(nk + 4):
            k0 = step * KS
            over = k0 >= D
            for tid in range(threads):
                chunk, lrow = tid & 7, tid >> 3
                k = chunk * 8 if over else k0 + chunk * 8
                k = min(k, D - 8)
                for i in range(hloads):
                    r = b0 + ((lrow & (BT - 1)) if partial else lrow + RPP * i)
                    r = min(r, B - 1)
                    out.append((r * D + k, 8))
    return out


SHAPES = [(128, 32, 256), (256, 32, 256), (128, 64, 256), (128, 128, 256), (256, 64, 512), (512, 32, 512)]


@pytest.mark.parametrize("D", [8, 16, 24, 56, 64, 72, 200])
@pytest.mark.parametrize("vrem", [1, 2, 129])
def test_every_load_stays_inside_its_buffer(D, vrem):
    for (VT, BT, threads), B in itertools.product(SHAPES, (1, 17, 33)):
        V = VT + vrem
        for off, n in w_addresses(D, V, VT, threads):
            assert 0 <= off and off + n <= V * D, ("W", D, V, VT, off)
        for off, n in h_addresses(D, B, BT, threads):
            assert 0 <= off and off + n <= B * D, ("H", D, B, BT, off)


def w4_addresses(D, V, VT, threads):
    """MXFP4 form of the kernel (K step 256 elements): byte offsets of every 16-byte load of codes and
    every 8-byte load of scale bytes."""
    KS4, WEPC, WCH = 256, 32, 8
    WRPP = threads // WCH
    NWL = VT // WRPP
    nk = D // KS4
    codes, scales = [], []
    for tile in range((V + VT - 1) // VT):
        tile_row0 = tile * VT
        for step in range(nk + 4):
            k0 = step * KS4
            over = k0 >= D
            for tid in range(threads):
                chunk, wrow = tid % WCH, tid // WCH
                k = chunk * WEPC if over else k0 + chunk * WEPC
                k = min(k, D - WEPC)
                for i in range(NWL):
                    row = min(tile_row0 + wrow + WRPP * i, V - 1)
                    row = tile_row0 if over else row
                    codes.append(((row * D + k) >> 1, 16))
                srow = min(tile_row0 + tid % VT, V - 1)
                srow = tile_row0 if over else srow
                kb = 0 if over else k0 >> 5
                scales.append((srow * (D >> 5) + kb, 8))
    return codes, scales


@pytest.mark.parametrize("D", [256, 512, 768, 4096])
@pytest.mark.parametrize("vrem", [1, 2, 129])
def test_every_load_of_the_mxfp4_form_stays_inside_its_buffer(D, vrem):
    for VT, threads in ((256, 256), (256, 512)):
        V = VT + vrem
        codes, scales = w4_addresses(D, V, VT, threads)
        for off, n in codes:
            assert 0 <= off and off + n <= V * D // 2 and off % 16 == 0, ("codes", D, V, off)
        for off, n in scales:
            assert 0 <= off and off + n <= V * D // 32 and off % 8 == 0, ("scales", D, V, off)
    # hidden rows: four 64-element sub-tiles per step, same clamping as the other forms
    for BT, threads, B in ((32, 256, 17), (64, 512, 40), (64, 512, 130)):
        RPP = threads // 8
        partial = BT < RPP
        hloads = 1 if partial else BT // RPP
        for bt in range((B + BT - 1) // BT):
            for step in range(D // 256 + 4):
                k0, over = step * 256, step * 256 >= D
                for hh in range(4):
                    for tid in range(threads):
                        chunk, lrow = tid & 7, tid >> 3
                        k = min(chunk * 8 if over else k0 + hh * 64 + chunk * 8, D - 8)
                        for i in range(hloads):
                            r = min(bt * BT + ((lrow & (BT - 1)) if partial else lrow + RPP * i), B - 1)
                            assert 0 <= r * D + k and r * D + k + 8 <= B * D
