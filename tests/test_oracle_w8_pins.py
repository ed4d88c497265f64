"""Pins for the oracle's FP8-weight path: the E4M3 decode against the format's definition and
against an independent library decode, and the path itself against the already pinned bf16 path
on weights that both can represent.  No GPU."""
import math

import numpy as np
import pytest

import fs_workloads as wl

torch = pytest.importorskip("torch")


def test_e4m3_decode_known_codes(orc):
    # OCP 8-bit floating point, E4M3: bias 7, no infinities, S.1111.111 is NaN, subnormals m/8 * 2^-6
    known = {0x00: 0.0, 0x38: 1.0, 0x3C: 1.5, 0x40: 2.0, 0x7E: 448.0, 0x08: 2.0 ** -6, 0x01: 2.0 ** -9,
             0x07: 7 * 2.0 ** -9, 0x77: 240.0, 0x78: 256.0, 0xB8: -1.0, 0xC0: -2.0, 0xFE: -448.0, 0x30: 0.5}
    for code, val in known.items():
        assert orc.e4m3_to_double(code) == val, hex(code)
    assert math.isnan(orc.e4m3_to_double(0x7F)) and math.isnan(orc.e4m3_to_double(0xFF))
    assert math.copysign(1.0, orc.e4m3_to_double(0x80)) == -1.0 and orc.e4m3_to_double(0x80) == 0.0


def test_e4m3_decode_equals_library_decode_for_all_codes(orc):
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = np.array([orc.e4m3_to_double(int(c)) for c in codes])
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], mine[ok])
    # every code is exactly representable in bf16 (what the kernel converts to)
    as_bf16 = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(mine[ok].astype(np.float32)))
    assert np.array_equal(as_bf16.astype(np.float64), mine[ok])


def test_quantiser_round_trips_and_bounds(orc):
    _, W = wl.make_small(D=64, V=50, B=1, data_seed=900)
    codes, scale = wl.quantize_e4m3(W)
    assert codes.dtype == np.uint8 and codes.shape == W.shape and scale.shape == (50,)
    deq = np.array([[orc.e4m3_to_double(int(c)) for c in row] for row in codes]) * scale[:, None]
    Wf = wl.bf16_bits_to_f32(W).astype(np.float64)
    assert not np.isnan(deq).any()
    # 3 mantissa bits: relative error <= 2^-4 for normals, absolute error <= scale * 2^-10 below them
    assert np.all(np.abs(deq - Wf) <= np.maximum(np.abs(Wf) * 2.0 ** -4, scale[:, None] * 2.0 ** -10) + 1e-30)
    assert np.all(np.abs(deq).max(axis=1) <= np.abs(Wf).max(axis=1) * (1 + 1e-6))


def test_w8_path_equals_bf16_path_on_decoded_weights(orc):
    H, W = wl.make_small(D=96, V=700, B=5, data_seed=901)
    codes, scale = wl.quantize_e4m3(W)
    tau = np.array([0.6, 0.9, 1.0, 1.3, 2.0], dtype=np.float32)
    # unit scales: the bf16 path on the decoded values is the same computation
    deq = np.array([[orc.e4m3_to_double(int(c)) for c in row] for row in codes], dtype=np.float32)
    Wb = wl.f32_to_bf16_bits(deq)
    a = orc.sample_w8(H, codes, None, tau, seed=17, row_offset=4, vocab_offset=128)
    b = orc.sample(H, Wb, tau, seed=17, row_offset=4, vocab_offset=128)
    assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(a["top1"], b["top1"])
    assert np.array_equal(a["idx2"], b["idx2"])
    # per-row scales multiply the logits: compare with numpy on the decoded matrix
    Y = orc.logits_w8(H, codes, scale)
    ref = wl.bf16_bits_to_f32(H).astype(np.float64) @ (deq.astype(np.float64) * scale[:, None].astype(np.float64)).T
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-12)
    c = orc.sample_w8(H, codes, scale, tau, seed=17)
    for r in range(5):
        i1, m1, _, _ = orc.gumbel_max_row(Y[r], float(tau[r]), 17, r)
        assert c["idx"][r] == i1 and c["top1"][r] == m1
        assert orc.score_at_w8(H, codes, scale, r, int(i1), float(tau[r]), 17, r, int(i1)) == m1
