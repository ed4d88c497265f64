"""GPU parity of the MXFP4-weight path (flash_sample_w4) against the oracle's fso_sample_w4."""
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


def test_on_chip_decode_of_every_code_and_scale(fs, orc):
    # every E2M1 code in every nibble position, under scales across the E8M0 range whose products
    # with the largest element (6) stay inside the bf16 range (e <= 252)
    scales = [0, 1, 2, 100, 120, 126, 127, 128, 133, 200, 250, 252]
    rng = np.random.default_rng(0)
    dwords = []
    for pos in range(8):
        for code in range(16):
            base = int(rng.integers(0, 2 ** 32, dtype=np.uint64))
            dwords.append((base & ~(0xF << (4 * pos))) | (code << (4 * pos)))
    dwords = np.array(dwords, dtype=np.uint32)
    for e in scales:
        sc = np.full(dwords.size, e, dtype=np.uint8)
        out = fs.flash_sample_mxfp4_decode(dev(dwords.view(np.uint8), np.uint8), dev(sc, np.uint8)).cpu().numpy()
        ref = np.array([[orc.e2m1_to_double((int(d) >> (4 * j)) & 15) * orc.e8m0_to_double(e) for j in range(8)]
                        for d in dwords]).reshape(-1)
        assert np.array_equal(out.astype(np.float64), ref), e
        assert np.array_equal(np.signbit(out), np.signbit(ref)), e


CASES = [(1, 512, 4096), (5, 512, 1189), (16, 4096, 2048 + 64), (9, 1024, 520), (3, 1536, 127), (2, 512, 5),
         (16, 3584, 700), (7, 8192, 300), (12, 7168, 400), (16, 5120, 130),
         # the tiled form: B > 16 (256 x 32 and 256 x 64 tiles, several batch tiles, ragged vocabulary tiles),
         # and small batches at hidden sizes the split-K form does not take (D % 512 != 0, D > 8192)
         (17, 512, 700), (32, 1024, 1189), (40, 512, 515), (64, 768, 300), (100, 256, 640), (130, 1024, 257),
         (4, 768, 520), (3, 256, 127), (5, 8704, 300), (33, 4096, 1000)]


@pytest.mark.parametrize("shape", CASES)
def test_w4_matches_oracle(fs, orc, shape):
    B, D, V = shape
    print(f"w4 parity shape={shape}", flush=True)
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=950 + B + V)
    codes, scales = wl.quantize_mxfp4(W)
    tau = np.linspace(0.6, 1.6, B).astype(np.float32)
    seeds = np.arange(B, dtype=np.uint64) + np.uint64(5)
    ref = orc.sample_w4(H, codes, scales, tau, row_seeds=seeds, row_offset=3, vocab_offset=256)
    lg = torch.empty((B, V), dtype=torch.float32, device="cuda")
    gi, gv = fs.flash_sample_w4(to_device_bf16(H), dev(codes, np.uint8), dev(scales, np.uint8), dev(tau, np.float32),
                                row_seeds=to_device_seeds(seeds), row_offset=3, vocab_offset=256, logits=lg)
    torch.cuda.synchronize()
    v = judge(orc, H, codes, tau, gi.cpu().numpy(), gv.cpu().numpy(), ref, row_seeds=seeds, row_offset=3,
              vocab_offset=256, w4_scales=scales)
    assert v.ok, (shape, str(v), v.failures[:3])
    Y = orc.logits_w4(H, codes, scales)
    assert np.max(np.abs(lg.cpu().numpy() - Y)) <= 2e-3


@pytest.mark.parametrize("wgs", [0, 1, 2])
def test_w4_every_kernel_form(fs, orc, wgs):
    # 16 K steps per wave (D <= 4096) and 32 (D % 1024 == 0, up to 8192); workgroups per CU automatic or forced
    for B, D, V in [(10, 1024, 700), (16, 4096, 300), (10, 6144, 700), (16, 8192, 300), (3, 512, 2000)]:
        print(f"w4 wgs/CU {wgs} B={B} D={D} V={V}", flush=True)
        H, W = wl.make_small(D=D, V=V, B=B, data_seed=970 + B)
        codes, scales = wl.quantize_mxfp4(W)
        tau = np.linspace(0.7, 1.5, B).astype(np.float32)
        ref = orc.sample_w4(H, codes, scales, tau, seed=9)
        gi, gv = fs.flash_sample_w4(to_device_bf16(H), dev(codes, np.uint8), dev(scales, np.uint8),
                                    dev(tau, np.float32), seed=9, flags=fs.FS_TUNE_WGS_PER_CU(wgs))
        torch.cuda.synchronize()
        v = judge(orc, H, codes, tau, gi.cpu().numpy(), gv.cpu().numpy(), ref, seed=9, w4_scales=scales)
        assert v.ok, (wgs, B, D, V, str(v), v.failures[:3])


def test_w4_at_llama_shape(fs, orc):
    w = wl.WORKLOADS["C2"]
    B = 16
    print("w4 parity at D=4096 V=128256 B=16", flush=True)
    H, W = wl.make_hidden(w, B), wl.make_weights(w)
    codes, scales = wl.quantize_mxfp4(W)
    tau = wl.make_temperature(w, B)
    seeds = wl.make_row_seeds(w, B)
    ref = orc.sample_w4(H, codes, scales, tau, row_seeds=seeds)
    gi, gv = fs.flash_sample_w4(to_device_bf16(H), dev(codes, np.uint8), dev(scales, np.uint8),
                                dev(tau, np.float32), row_seeds=to_device_seeds(seeds))
    torch.cuda.synchronize()
    v = judge(orc, H, codes, tau, gi.cpu().numpy(), gv.cpu().numpy(), ref, row_seeds=seeds, w4_scales=scales)
    assert v.ok, (str(v), v.failures[:3])


def test_w4_at_llama_shape_larger_batches(fs, orc):
    # the tiled form at full size, every row judged
    w = wl.WORKLOADS["C2"]
    W = wl.make_weights(w)
    codes, scales = wl.quantize_mxfp4(W)
    cd, sd = dev(codes, np.uint8), dev(scales, np.uint8)
    for B in (32, 64):
        print(f"w4 parity at D=4096 V=128256 B={B}", flush=True)
        H = wl.make_hidden(w, B)
        tau = wl.make_temperature(w, B)
        seeds = wl.make_row_seeds(w, B)
        ref = orc.sample_w4(H, codes, scales, tau, row_seeds=seeds)
        gi, gv = fs.flash_sample_w4(to_device_bf16(H), cd, sd, dev(tau, np.float32), row_seeds=to_device_seeds(seeds))
        torch.cuda.synchronize()
        v = judge(orc, H, codes, tau, gi.cpu().numpy(), gv.cpu().numpy(), ref, row_seeds=seeds, w4_scales=scales)
        print(f"[parity] w4 C2 B={B}: {v}", flush=True)
        assert v.ok and v.rows == B, (B, str(v), v.failures[:3])


def test_w4_shapes_outside_the_kernel_are_refused(fs):
    tau = torch.ones(17, device="cuda")
    for B, D in [(17, 288), (4, 160), (4, 4608 + 32)]:          # hidden sizes that are not whole K steps of 256
        H = torch.zeros((B, D), dtype=torch.bfloat16, device="cuda")
        W4 = torch.zeros((256, D // 2), dtype=torch.uint8, device="cuda")
        S = torch.zeros((256, D // 32), dtype=torch.uint8, device="cuda")
        with pytest.raises(fs.FlashSampleError) as e:
            fs.flash_sample_w4(H, W4, S, tau[:B])
        assert e.value.status == fs.FS_ERR_UNSUPPORTED, (B, D)
