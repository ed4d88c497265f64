"""GPU parity of the FP8-weight path (flash_sample_w8) against the oracle's fso_sample_w8."""
import numpy as np
import pytest

import fs_workloads as wl
from tests.parity import judge, to_device_bf16, to_device_seeds

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def fs():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    import paper_2603_15854_amd as fs
    fs.lib()
    return fs


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).cuda()


def test_on_chip_decode_of_every_code(fs, orc):
    codes = np.arange(256, dtype=np.uint8)
    out = fs.flash_sample_e4m3_decode(dev(codes, np.uint8)).cpu().numpy()
    ref = np.array([orc.e4m3_to_double(int(c)) for c in codes])
    assert np.array_equal(np.isnan(out), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(out[ok].astype(np.float64), ref[ok])
    assert np.array_equal(np.signbit(out[ok]), np.signbit(ref[ok]))


CASES = [(1, 256, 4096), (5, 512, 1189), (16, 4096, 2048 + 64), (9, 2064, 520), (3, 48, 127), (2, 16, 5),
         (16, 1040, 3000), (7, 4096, 300),
         # tiled kernel: wide hidden sizes at small B, and B > 16 with each batch-tile width, ragged V and K
         (4, 8192, 700), (12, 7184, 300), (20, 528, 1100), (40, 1040, 1300), (70, 256, 3000), (150, 1072, 700),
         (300, 256, 1000)]


@pytest.mark.parametrize("shape", CASES)
@pytest.mark.parametrize("scaled", [True, False])
def test_w8_matches_oracle(fs, orc, shape, scaled):
    B, D, V = shape
    print(f"w8 parity shape={shape} scaled={scaled}", flush=True)
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=800 + B + V)
    codes, scale = wl.quantize_e4m3(W)
    if not scaled:
        scale = None
    tau = np.linspace(0.6, 1.6, B).astype(np.float32)
    seeds = np.arange(B, dtype=np.uint64) + np.uint64(11)
    ref = orc.sample_w8(H, codes, scale, tau, row_seeds=seeds, row_offset=3, vocab_offset=256)
    lg = torch.empty((B, V), dtype=torch.float32, device="cuda")
    gi, gv = fs.flash_sample_w8(to_device_bf16(H), dev(codes, np.uint8), None if scale is None else dev(scale, np.float32),
                                dev(tau, np.float32), row_seeds=to_device_seeds(seeds), row_offset=3,
                                vocab_offset=256, logits=lg)
    torch.cuda.synchronize()
    v = judge(orc, H, codes, tau, gi.cpu().numpy(), gv.cpu().numpy(), ref, row_seeds=seeds, row_offset=3,
              vocab_offset=256, w8_scale=scale)
    assert v.ok, (shape, scaled, str(v), v.failures[:3])
    Y = orc.logits_w8(H, codes, scale)
    # 2e-3 absolute on logits of order one; without the scales the terms are up to 448 times larger,
    # so the budget there is the fp32 accumulation bound 8 eps sum_d |h_d w_d|
    deq = np.abs(np.array([orc.e4m3_to_double(c) for c in range(256)]))[codes]
    if scale is not None:
        deq = deq * scale[:, None]
    mag = np.abs(wl.bf16_bits_to_f32(H).astype(np.float64)) @ deq.T
    assert np.all(np.abs(lg.cpu().numpy() - Y) <= 2e-3 + 8 * 2.0 ** -24 * mag)


def test_w8_at_llama_shape(fs, orc):
    # the bandwidth-bound decode shape, every row checked against the oracle
    w = wl.WORKLOADS["C2"]
    B = 16
    print("w8 parity at D=4096 V=128256 B=16", flush=True)
    H, W = wl.make_hidden(w, B), wl.make_weights(w)
    codes, scale = wl.quantize_e4m3(W)
    tau = wl.make_temperature(w, B)
    seeds = wl.make_row_seeds(w, B)
    ref = orc.sample_w8(H, codes, scale, tau, row_seeds=seeds)
    gi, gv = fs.flash_sample_w8(to_device_bf16(H), dev(codes, np.uint8), dev(scale, np.float32),
                                dev(tau, np.float32), row_seeds=to_device_seeds(seeds))
    torch.cuda.synchronize()
    v = judge(orc, H, codes, tau, gi.cpu().numpy(), gv.cpu().numpy(), ref, row_seeds=seeds, w8_scale=scale)
    assert v.ok, (str(v), v.failures[:3])


@pytest.mark.parametrize("tune", [-1, 1, 2, 3, 4, 5, 6, 7, 8, 10, 12])
def test_w8_every_kernel_choice(fs, orc, tune):
    # -1: the split-K kernel forced; others: the tile shapes of the tiled kernel (codes kept in LDS when
    # D % 128 == 0, widened at park time on the two-per-CU shapes otherwise)
    shapes = [(10, 528, 1100), (16, 2048, 700), (7, 8192, 300)] if tune < 0 else \
        [(20, 528, 1100), (70, 256, 1500), (150, 1152, 700), (33, 48, 513), (40, 192, 600)]
    for B, D, V in shapes:
        print(f"w8 tune {tune} B={B} D={D} V={V}", flush=True)
        H, W = wl.make_small(D=D, V=V, B=B, data_seed=850 + B)
        codes, scale = wl.quantize_e4m3(W)
        tau = np.linspace(0.7, 1.5, B).astype(np.float32)
        ref = orc.sample_w8(H, codes, scale, tau, seed=9)
        flags = fs.FS_VARIANT(fs.FS_VARIANT_SPLITK) if tune < 0 else \
            fs.FS_VARIANT(fs.FS_VARIANT_TILED2) | fs.FS_TUNE_TILE_SHAPE(tune)
        gi, gv = fs.flash_sample_w8(to_device_bf16(H), dev(codes, np.uint8), dev(scale, np.float32),
                                    dev(tau, np.float32), seed=9, flags=flags)
        torch.cuda.synchronize()
        v = judge(orc, H, codes, tau, gi.cpu().numpy(), gv.cpu().numpy(), ref, seed=9, w8_scale=scale)
        assert v.ok, (tune, B, D, V, str(v), v.failures[:3])


def test_w8_shapes_outside_the_kernel_are_refused(fs):
    H = torch.zeros((17, 256), dtype=torch.bfloat16, device="cuda")
    W8 = torch.zeros((512, 256), dtype=torch.uint8, device="cuda")
    tau = torch.ones(17, device="cuda")
    with pytest.raises(fs.FlashSampleError) as e:    # split-K variant asked for B > 16
        fs.flash_sample_w8(H, W8, None, tau, flags=fs.FS_VARIANT(2))
    assert e.value.status == fs.FS_ERR_UNSUPPORTED
    with pytest.raises(fs.FlashSampleError) as e:    # D % 16 != 0
        fs.flash_sample_w8(H[:4, :248].contiguous(), W8[:, :248].contiguous(), None, tau[:4])
    assert e.value.status == fs.FS_ERR_SHAPE


@pytest.mark.parametrize("shape", [(20, 16, 200), (40, 64, 3), (130, 128, 1), (33, 192, 129)])
def test_w8_degenerate_shapes_on_the_tiled_kernels(fs, orc, shape):
    B, D, V = shape
    print(f"w8 degenerate shape {shape}", flush=True)
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=880 + B + V)
    codes, scale = wl.quantize_e4m3(W)
    tau = np.linspace(0.7, 1.5, B).astype(np.float32)
    ref = orc.sample_w8(H, codes, scale, tau, seed=4)
    gi, gv = fs.flash_sample_w8(to_device_bf16(H), dev(codes, np.uint8), dev(scale, np.float32),
                                dev(tau, np.float32), seed=4)
    torch.cuda.synchronize()
    v = judge(orc, H, codes, tau, gi.cpu().numpy(), gv.cpu().numpy(), ref, seed=4, w8_scale=scale)
    assert v.ok, (shape, str(v), v.failures[:3])
