"""Pins for the oracle's MXFP4-weight path: element and scale decode against the format's
definition, the block quantiser's error bound, and the path itself against the already pinned bf16
path on the dequantised weights.  No GPU."""
import math

import numpy as np

import fs_workloads as wl


def test_e2m1_and_e8m0_decode(orc):
    # OCP microscaling formats: FP4 E2M1 magnitudes and the E8M0 power-of-two scale
    mags = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    for c in range(8):
        assert orc.e2m1_to_double(c) == mags[c]
        assert orc.e2m1_to_double(c | 8) == -mags[c]
    assert math.copysign(1.0, orc.e2m1_to_double(8)) == -1.0
    # the same magnitudes from the field definition: bias 1, one mantissa bit, subnormal 0.5
    for c in range(8):
        e, m = c >> 1, c & 1
        ref = (m * 0.5) if e == 0 else (1 + m * 0.5) * 2.0 ** (e - 1)
        assert orc.e2m1_to_double(c) == ref
    assert orc.e8m0_to_double(127) == 1.0 and orc.e8m0_to_double(128) == 2.0
    assert orc.e8m0_to_double(0) == 2.0 ** -127 and orc.e8m0_to_double(254) == 2.0 ** 127
    assert math.isnan(orc.e8m0_to_double(255))


def _dequant(orc, codes, scales):
    V, half = codes.shape
    lo = np.array([orc.e2m1_to_double(c) for c in range(16)])
    el = np.empty((V, half * 2))
    el[:, 0::2] = lo[codes & 15]
    el[:, 1::2] = lo[codes >> 4]
    sc = np.array([orc.e8m0_to_double(e) if e != 255 else np.nan for e in range(256)])[scales]
    return el * np.repeat(sc, 32, axis=1)


def test_quantiser_layout_and_error_bound(orc):
    _, W = wl.make_small(D=128, V=40, B=1, data_seed=910)
    codes, scales = wl.quantize_mxfp4(W)
    assert codes.shape == (40, 64) and scales.shape == (40, 4) and codes.dtype == np.uint8
    deq = _dequant(orc, codes, scales)
    Wf = wl.bf16_bits_to_f32(W).astype(np.float64)
    amax = np.abs(Wf.reshape(40, 4, 32)).max(axis=2)
    step = np.repeat(np.exp2(np.floor(np.log2(amax)) - 2), 32, axis=1)   # one unit of the block's grid
    # nearest-grid rounding: at most one grid unit (between 4 and 6) or saturation from < 8 to 6
    assert np.all(np.abs(deq - Wf) <= 2.0 * step + 1e-30)
    assert np.all(np.sign(deq) * np.sign(Wf) >= 0)
    # a hand-made block: element 2j in the low nibble of byte j
    Wb = wl.f32_to_bf16_bits(np.array([[6.0, -0.5] + [0.0] * 30], dtype=np.float32))
    c, s = wl.quantize_mxfp4(Wb)
    assert int(s[0, 0]) == 127 and int(c[0, 0]) == (7 | (9 << 4)) and not c[0, 1:].any()


def test_w4_path_equals_bf16_path_on_dequantised_weights(orc):
    H, W = wl.make_small(D=96, V=600, B=4, data_seed=911)
    codes, scales = wl.quantize_mxfp4(W)
    deq = _dequant(orc, codes, scales)
    Wb = wl.f32_to_bf16_bits(deq.astype(np.float32))
    assert np.array_equal(wl.bf16_bits_to_f32(Wb).astype(np.float64), deq)      # exactly bf16 values
    tau = np.array([0.6, 1.0, 1.3, 2.0], dtype=np.float32)
    a = orc.sample_w4(H, codes, scales, tau, seed=19, row_offset=2, vocab_offset=64)
    b = orc.sample(H, Wb, tau, seed=19, row_offset=2, vocab_offset=64)
    assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(a["idx2"], b["idx2"])
    assert np.allclose(a["top1"], b["top1"], rtol=1e-13, atol=1e-13)
    Y = orc.logits_w4(H, codes, scales)
    ref = wl.bf16_bits_to_f32(H).astype(np.float64) @ deq.T
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-12)
    for r in range(4):
        assert orc.score_at_w4(H, codes, scales, r, int(a["idx"][r]) - 64, float(tau[r]), 19, 2 + r,
                               int(a["idx"][r])) == a["top1"][r]
