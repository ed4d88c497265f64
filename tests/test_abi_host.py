"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and its byte model matches
the paper's IO cost model."""
import os
import re

import pytest

import fs_io_model as iom
import paper_2603_15854_amd as fs
from paper_2603_15854_amd import measure as fsm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "flash_sample.h")
MEASURE_HEADER = os.path.join(ROOT, "include", "flash_sample_measure.h")
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

FAKE = 0x7F0000001000  # an aligned, never dereferenced address: the checks under test return first


def _declared_symbols(header):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flash_[a-z0-9_]+|fs_status_string)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = fs.lib()
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["flash_sample.h", "flash_sample_measure.h"]
    for header, exports in ((HEADER, fs.EXPORTS), (MEASURE_HEADER, fs.MEASURE_EXPORTS)):
        declared = _declared_symbols(header)
        assert declared, "no declarations found in the header"
        for name in declared:
            assert hasattr(L, name), name
        assert sorted(exports) == declared        # the binding covers the same set


def test_tile_and_workspace_arithmetic():
    assert fs.FS_VOCAB_TILE == 128
    assert fs.flash_sample_num_tiles(4096) == 32          # config 1: T = 32
    assert fs.flash_sample_num_tiles(128256) == 1002
    assert fs.flash_sample_num_tiles(152064) == 1188
    assert fs.flash_sample_num_tiles(129280) == 1010
    assert fs.flash_sample_num_tiles(129) == 2 and fs.flash_sample_num_tiles(1) == 1
    assert fs.flash_sample_num_tiles(0) == 0
    # candidates: one fp32 + one int32 per (row, tile), two 256-byte aligned parts
    assert fs.flash_sample_workspace_bytes(16, 128256) == 2 * 64256          # 16*1002*4 = 64128 -> 64256
    assert fs.flash_sample_workspace_bytes(1, 4096) == 2 * 256
    assert fs.flash_sample_workspace_bytes(0, 4096) == 0


def test_status_strings():
    seen = set()
    for code in range(0, 9):
        s = fs.fs_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert fs.fs_status_string(99) == "unknown status"


def test_bad_arguments_are_rejected_before_any_device_work():
    L = fs.lib()

    def ex(hidden=FAKE, W=FAKE, B=4, D=256, V=4096, tau=FAKE, row_offset=0, vocab_offset=0,
           out_idx=FAKE, out_val=FAKE, ws=FAKE + 0x100000, ws_bytes=1 << 20, flags=0):
        return L.flash_sample_ex(hidden, W, B, D, V, tau, 0, None, row_offset, vocab_offset, out_idx,
                                 out_val, ws, ws_bytes, None, flags)

    assert ex(B=0) == fs.FS_OK                                  # empty batch: successful no-op
    assert ex(B=0, hidden=None, W=None, tau=None, out_idx=None, out_val=None, ws=None, ws_bytes=0) == fs.FS_OK
    assert ex(B=-1) == fs.FS_ERR_SHAPE
    assert ex(D=0) == fs.FS_ERR_SHAPE and ex(V=0) == fs.FS_ERR_SHAPE
    assert ex(D=250) == fs.FS_ERR_SHAPE                         # D % 8 != 0
    assert ex(vocab_offset=-1) == fs.FS_ERR_SHAPE
    assert ex(vocab_offset=2**31 - 1 - 4095) == fs.FS_ERR_SHAPE  # vocab_offset + V overflows int32
    assert ex(row_offset=-5) == fs.FS_ERR_SHAPE
    assert ex(hidden=None) == fs.FS_ERR_NULL and ex(W=None) == fs.FS_ERR_NULL
    assert ex(tau=None) == fs.FS_ERR_NULL and ex(out_idx=None) == fs.FS_ERR_NULL
    assert ex(out_val=None) == fs.FS_ERR_NULL
    assert ex(hidden=FAKE + 8) == fs.FS_ERR_ALIGN and ex(W=FAKE + 2) == fs.FS_ERR_ALIGN
    assert ex(out_idx=FAKE + 2) == fs.FS_ERR_ALIGN
    assert ex(ws=None) == fs.FS_ERR_WORKSPACE
    assert ex(ws=FAKE + 0x100010) == fs.FS_ERR_WORKSPACE        # not 256-byte aligned
    assert ex(ws_bytes=fs.flash_sample_workspace_bytes(4, 4096) - 1) == fs.FS_ERR_WORKSPACE

    # the plain entry point, the stages and the unfused path share the checks
    assert L.flash_sample(None, FAKE, 1, 256, 4096, FAKE, 0, FAKE, FAKE) == fs.FS_ERR_NULL
    assert L.flash_sample(FAKE, FAKE, 1, 252, 4096, FAKE, 0, FAKE, FAKE) == fs.FS_ERR_SHAPE
    assert L.flash_sample(FAKE, FAKE, 0, 256, 4096, FAKE, 0, FAKE, FAKE) == fs.FS_OK
    assert L.flash_sample_stage1(FAKE, FAKE, 1, 256, 4096, FAKE, 0, None, 0, 0, None, None, None, None, 0) == fs.FS_ERR_NULL
    assert L.flash_sample_stage1(FAKE, FAKE, 1, 256, 4096, FAKE, 0, None, 0, 0, FAKE, None, None, None, 0) == fs.FS_ERR_NULL
    assert L.flash_sample_stage2(None, FAKE, 1, 32, FAKE, FAKE, None) == fs.FS_ERR_NULL
    assert L.flash_sample_stage2(FAKE, FAKE, 1, 0, FAKE, FAKE, None) == fs.FS_ERR_SHAPE
    assert L.flash_sample_stage2(FAKE, FAKE, 0, 32, FAKE, FAKE, None) == fs.FS_OK
    assert L.flash_sample_unfused(FAKE, FAKE, 1, 256, 4096, FAKE, 0, None, 0, 0, None, FAKE, FAKE,
                                  FAKE, 1 << 20, None, 0) == fs.FS_ERR_NULL
    assert L.flash_lm_head_logits(FAKE, FAKE, 1, 256, 4096, None, None, 0) == fs.FS_ERR_NULL
    assert L.flash_gumbel_argmax_logits(FAKE, 1, 0, FAKE, 0, None, 0, 0, FAKE, FAKE, FAKE, 1 << 20, None) == fs.FS_ERR_SHAPE
    assert L.flash_sample_noise(0, 0, 0, -1, FAKE, None) == fs.FS_ERR_SHAPE
    assert L.flash_sample_noise(0, 0, 0, 0, None, None) == fs.FS_OK
    assert L.flash_sample_gumbel_transform(None, 4, FAKE, None, 0) == fs.FS_ERR_NULL
    assert L.flash_sample_gumbel_transform(FAKE, 4, FAKE, None, fs.FS_FLAG_GREEDY) == fs.FS_ERR_UNSUPPORTED
    assert L.flash_measure_stream_probe(None, FAKE, 24, None, None) == fs.FS_ERR_SHAPE
    assert L.flash_measure_stream_probe(None, None, 32, None, None) == fs.FS_ERR_NULL
    # unknown flag bits and retired variant numbers
    for bad in (0x4, 0x40, fs.FS_VARIANT(1), fs.FS_VARIANT(3), fs.FS_VARIANT(99), 1 << 20):
        assert ex(flags=bad) == fs.FS_ERR_UNSUPPORTED, hex(bad)

    # the entry point on the built-in scratch: same checks, plus its size limit (before any device work)
    def static(B=4, V=4096, hidden=FAKE, out_idx=FAKE, D=256):
        return L.flash_sample_static(hidden, FAKE, B, D, V, FAKE, 0, None, 0, 0, out_idx, FAKE, None, 0)

    assert static(B=0) == fs.FS_OK
    assert static(hidden=None) == fs.FS_ERR_NULL and static(D=252) == fs.FS_ERR_SHAPE
    assert fs.flash_sample_workspace_bytes(512, 129280) <= fs.FS_STATIC_SCRATCH_BYTES
    Bmax = fs.FS_STATIC_SCRATCH_BYTES // (8 * 1002)
    assert fs.flash_sample_workspace_bytes(Bmax + 1, 128256) > fs.FS_STATIC_SCRATCH_BYTES
    assert static(B=Bmax + 1, V=128256) == fs.FS_ERR_SCRATCH_LIMIT
    assert static(B=4, V=2**31 - 2) == fs.FS_ERR_SCRATCH_LIMIT
    assert "scratch" in fs.fs_status_string(fs.FS_ERR_SCRATCH_LIMIT)

    # FP8 weights
    def w8(B=4, D=256, out_idx=FAKE, ws=FAKE + 0x100000, flags=0):
        return L.flash_sample_w8(FAKE, FAKE, None, B, D, 4096, FAKE, 0, None, 0, 0, None, out_idx, FAKE,
                                 ws, 1 << 20, None, flags)

    assert w8(B=0) == fs.FS_OK
    assert w8(D=248) == fs.FS_ERR_SHAPE                         # D % 16 != 0
    assert w8(out_idx=None) == fs.FS_ERR_NULL
    assert w8(ws=None) == fs.FS_ERR_WORKSPACE
    assert L.flash_sample_e4m3_decode(FAKE, 12, FAKE, None) == fs.FS_ERR_SHAPE
    assert L.flash_sample_e4m3_decode(None, 16, FAKE, None) == fs.FS_ERR_NULL
    assert L.flash_sample_e4m3_decode(FAKE, 0, None, None) == fs.FS_OK

    # grouped variants
    def gr(B=4, V=4096, vocab_offset=0, gt=2, mode=0, out_idx=FAKE, ws=FAKE + 0x100000, ws_bytes=1 << 20):
        return L.flash_sample_grouped(FAKE, FAKE, B, 256, V, FAKE, 0, None, 0, vocab_offset, None, None, 0,
                                      gt, mode, out_idx, None, None, None, ws, ws_bytes, None, 0)

    assert gr(B=0) == fs.FS_OK
    assert gr(gt=0) == fs.FS_ERR_SHAPE and gr(mode=2) == fs.FS_ERR_SHAPE
    assert gr(vocab_offset=128) == fs.FS_ERR_SHAPE              # not a multiple of the group size
    assert gr(vocab_offset=256, B=0) == fs.FS_OK
    assert gr(out_idx=None) == fs.FS_ERR_NULL
    assert gr(ws_bytes=fs.flash_sample_full_workspace_bytes(4, 4096) - 1) == fs.FS_ERR_WORKSPACE
    assert fs.flash_sample_num_groups(4096, 1) == 32 and fs.flash_sample_num_groups(4097, 8) == 5
    assert fs.flash_sample_num_groups(0, 1) == 0 and fs.flash_sample_num_groups(128, 0) == 0
    assert L.flash_group_choose(FAKE, FAKE, 0, 8, 0, 0, None, 0, 0, FAKE, None, None) == fs.FS_OK
    assert L.flash_group_choose(None, FAKE, 2, 8, 0, 0, None, 0, 0, FAKE, None, None) == fs.FS_ERR_NULL
    assert L.flash_group_choose(FAKE, FAKE, 2, 0, 0, 0, None, 0, 0, FAKE, None, None) == fs.FS_ERR_SHAPE
    assert L.flash_group_choose(FAKE, FAKE, 2, 8, 3, 0, None, 0, 0, FAKE, None, None) == fs.FS_ERR_SHAPE
    assert L.flash_group_choose(FAKE, FAKE, 2, 8, 0, 0, None, 0, -1, FAKE, None, None) == fs.FS_ERR_SHAPE


def test_topk_arguments_and_workspace_without_a_device():
    L = fs.lib()
    wsb = fs.flash_sample_topk_workspace_bytes

    def tk(B=4, D=256, V=4096, k=8, top_p=1.0, mode=0, tau=FAKE, out_idx=FAKE, out_val=FAKE, ws=FAKE + 0x100000,
           ws_bytes=1 << 24, flags=0, fused=True, logits=FAKE):
        common = (FAKE, FAKE, B, D, V, tau, 0, None, 0, 0, k, top_p, mode)
        tail = (out_idx, out_val, None, None, None, ws, ws_bytes, None, flags)
        return L.flash_sample_topk(*common, *tail) if fused else L.flash_sample_topk_unfused(*common, logits, *tail)

    for fused in (True, False):
        assert tk(B=0, fused=fused) == fs.FS_OK
        assert tk(k=0, fused=fused) == fs.FS_ERR_SHAPE and tk(k=fs.FS_TOPK_MAX_K + 1, fused=fused) == fs.FS_ERR_SHAPE
        assert tk(top_p=0.0, fused=fused) == fs.FS_ERR_SHAPE and tk(top_p=1.01, fused=fused) == fs.FS_ERR_SHAPE
        assert tk(top_p=float("nan"), fused=fused) == fs.FS_ERR_SHAPE
        assert tk(mode=2, fused=fused) == fs.FS_ERR_SHAPE
        assert tk(mode=fs.FS_TOPK_GUMBEL, top_p=0.9, fused=fused) == fs.FS_ERR_SHAPE     # the candidates are the draw
        assert tk(flags=fs.FS_FLAG_GREEDY, fused=fused) == fs.FS_ERR_UNSUPPORTED
        assert tk(tau=None, fused=fused) == fs.FS_ERR_NULL and tk(out_idx=None, fused=fused) == fs.FS_ERR_NULL
        assert tk(out_val=FAKE + 2, fused=fused) == fs.FS_ERR_ALIGN
        assert tk(ws=None, fused=fused) == fs.FS_ERR_WORKSPACE
        assert tk(D=252, fused=fused) == fs.FS_ERR_SHAPE
    assert tk(ws_bytes=wsb(4, 4096, 8) - 1) == fs.FS_ERR_WORKSPACE   # (the form over stored logits needs less)
    assert tk(D=200) == fs.FS_ERR_UNSUPPORTED                  # the fused form takes whole K steps only
    assert tk(fused=False, logits=None) == fs.FS_ERR_NULL
    # workspace: zero for impossible arguments, monotone in B, the fused candidates dominate
    assert wsb(0, 4096, 8) == 0 and wsb(4, 4096, 0) == 0 and wsb(4, 4096, 65) == 0
    assert wsb(4, 4096, 8) >= 4 * 32 * 8 * 8                    # B x T x m words
    assert wsb(256, 128256, 50) >= 256 * 1002 * 4 * 8 and wsb(256, 128256, 50) < 32 << 20
    assert wsb(16, 128256, 50) >= 16 * 1002 * 8 * 8
    assert wsb(8, 128256, 50) <= wsb(16, 128256, 50) <= wsb(32, 128256, 50) * 2


def test_kernel_choice_by_shape():
    # the launcher's rule: split-K while the hidden slice of a wave fits its registers, else the
    # tile shape with the cheapest busiest CU, ceil(workgroups / CUs) * (rows + columns), finer on ties
    kc = fsm.flash_measure_kernel_choice
    assert [kc(B, 4096, 128256) for B in (1, 16)] == [0, 0]
    assert [kc(B, 4096, 128256) for B in (17, 32, 64, 128, 129, 256, 512)] == [6, 6, 7, 10, 12, 12, 12]
    assert kc(16, 8192, 128256) == 6 and kc(1, 7168, 129280) == 6          # wide hidden sizes: tiled
    assert kc(128, 8192, 128256) == 13 and kc(128, 7168, 129280) == 13      # ... and direct-to-LDS loads at B <= 128
    # the choices measured fastest on the machine (D = 4096, 256 CUs)
    assert [kc(32, 4096, V) for V in (32000, 50304, 100352, 152064, 201088)] == [1, 8, 6, 1, 6]
    assert [kc(64, 4096, V) for V in (32000, 50304, 100352, 152064)] == [5, 2, 7, 5]
    assert [kc(128, 4096, V) for V in (32000, 50304, 100352, 152064, 201088, 256000)] == [4, 3, 10, 4, 10, 10]
    assert [kc(256, 4096, V) for V in (32000, 50304, 100352, 152064, 201088)] == [13, 12, 12, 12, 12]
    # above 128 rows: 256 x 128 tiles where the last 256-row batch tile would be at most half full
    assert [kc(B, 4096, 128256) for B in (160, 320, 384, 512, 640, 768)] == [12, 13, 13, 12, 12, 12]
    assert [kc(B, 4096, 32000) for B in (160, 320, 512, 768)] == [13, 12, 12, 13]
    assert [kc(B, 520, 128256) for B in (20, 64, 200)] == [8, 5, 4]        # D % 64 != 0
    assert kc(4, 4096, 1000) == 0 and kc(40, 4096, 1000) == 5              # a handful of tiles: fine shapes
    assert kc(0, 4096, 10) == -1 and kc(4, 4100, 10) == -1 and kc(4, 4096, 10, 0) == -1


def test_io_model_matches_the_papers_predicted_overheads():
    # appendix table "Predicted vs. measured overhead of storing logits to HBM": 2B/D in percent
    rows = []
    with open(os.path.join(GOLDEN, "io_model.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                D, V, B, pct = line.split()
                rows.append((int(D), int(V), int(B), float(pct)))
    assert len(rows) == 12
    for D, V, B, pct in rows:
        model = (iom.io_model_speedup_elements(B, D, V) - 1.0) * 100.0
        approx = 200.0 * B / D                                   # the printed column is 2B/D
        assert abs(approx - pct) <= 0.0051, (D, V, B, approx, pct)
        # the exact ratio 1 + 2/(D/B + D/V + 1/V) differs from it only by the D/V and 1/V terms
        exact = 200.0 / (D / B + D / V + 1.0 / V)
        assert abs(model - exact) < 1e-9
        assert 0 < approx - model < approx * 1.01 * B / V
    # byte form used by the benchmark: fp32 logits double the element-count overhead (4B/D)
    B, D, V = 16, 4096, 128256
    fused, unfused = iom.io_model_bytes(B, D, V, True), iom.io_model_bytes(B, D, V, False)
    assert fused == 2 * V * D + 2 * B * D + 16 * B * 1002 + 8 * B
    assert abs((unfused - fused) / fused - 4 * B / D) < 2e-3


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(fs, "_lib", None)
    monkeypatch.setattr(fs, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        fs.lib()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "ONE GPU" in res.stderr and res.stdout.strip() == ""
