"""GPU parity of the grouped variants (flash_sample_grouped, flash_group_choose) against the
oracle's fso_sample_grouped on the same seeded inputs, plus the sampling law on the GPU."""
import numpy as np
import pytest

import fs_workloads as wl
from tests.parity import judge_grouped, lse_tol, to_device_bf16, to_device_seeds
from tests.test_oracle_pins import _chi2_ok

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

PAR, ONL = 0, 1


@pytest.fixture(scope="module")
def fs():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    import paper_2603_15854_amd as fs
    fs.lib()
    return fs


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).cuda()


def dev_words(words):
    return None if words is None else torch.from_numpy(np.ascontiguousarray(words).view(np.int32)).cuda()


def run_grouped(fs, H, W, tau, gt, mode, *, seed=0, row_seeds=None, bias=None, words=None, **kw):
    idx, lse, gl, gs = fs.flash_sample_grouped(
        to_device_bf16(H), to_device_bf16(W), dev(tau, np.float32), group_tiles=gt, mode=mode, seed=seed,
        row_seeds=to_device_seeds(row_seeds), bias=None if bias is None else dev(bias, np.float32),
        allowed=dev_words(words), want_groups=True, **kw)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), lse.cpu().numpy(), gl.cpu().numpy(), gs.cpu().numpy()


CASES = [
    # (B, D, V, group_tiles): split-K and tiled stage-1 kernels, ragged last tile and last group,
    # one group in all, more groups than the 256 threads of the choice kernel
    (5, 512, 1189, 1), (5, 512, 1189, 3), (16, 4096, 2048 + 64, 4), (1, 256, 4096, 1), (3, 24, 127, 1),
    (2, 8, 5, 2), (9, 256, 128 * 300 + 17, 1), (4, 64, 128 * 700, 2), (40, 1032, 1300, 2),
    (100, 264, 640, 5), (130, 512, 1515, 1), (300, 256, 1000, 100),
]


@pytest.mark.parametrize("shape", CASES)
@pytest.mark.parametrize("mode", [PAR, ONL])
def test_grouped_matches_oracle(fs, orc, shape, mode):
    B, D, V, gt = shape
    print(f"grouped parity shape={shape} mode={mode}", flush=True)
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=400 + B + V)
    rng = np.random.default_rng(B * 11 + V)
    tau = np.linspace(0.6, 1.6, B).astype(np.float32)
    bias = rng.normal(0, 1.0, V).astype(np.float32)
    allowed = rng.random((B, V)) < 0.7
    allowed[:, V // 2] = True
    if V > 256:
        allowed[0, 128:256] = False            # row 0: tile 1 has no mass
    if B > 2:
        allowed[2, :] = False                  # a row with no mass at all
    words = orc.pack_allowed(allowed)
    row_seeds = (np.arange(B, dtype=np.uint64) * np.uint64(7919) + np.uint64(3))
    g = 128 * gt
    ref = orc.sample_grouped(H, W, tau, g, mode, row_seeds=row_seeds, bias=bias, allowed_words=words)
    gi, gl, gL, gz = run_grouped(fs, H, W, tau, gt, mode, row_seeds=row_seeds, bias=bias, words=words)
    assert gL.shape == ref["L"].shape == (B, fs.flash_sample_num_groups(V, gt))
    v = judge_grouped(orc, mode, ref, H, W, tau, gi, gl, gL, gz, g=g, row_seeds=row_seeds, bias=bias,
                      allowed_words=words)
    assert v.ok, (shape, mode, str(v), v.failures[:3])
    assert v.near_ties <= max(2, B // 10), str(v)
    if B > 2:
        assert gi[2] == -1 and gl[2] == -np.inf


def test_one_group_is_the_default_draw(fs, orc):
    # a single group covering the whole vocabulary: both variants return the plain Gumbel-max pick
    B, D, V = 12, 512, 1000
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=420)
    tau = np.full(B, 0.8, dtype=np.float32)
    Hd, Wd, td = to_device_bf16(H), to_device_bf16(W), dev(tau, np.float32)
    a_i, _ = fs.flash_sample_ex(Hd, Wd, td, seed=9)
    for mode in (PAR, ONL):
        g_i, g_l, _, _ = fs.flash_sample_grouped(Hd, Wd, td, group_tiles=8, mode=mode, seed=9)
        torch.cuda.synchronize()
        assert torch.equal(a_i, g_i)


def test_vocabulary_shards_as_groups(fs, orc):
    # distributed variant on one GPU: every shard reports (L_k, z_k) with one group per shard,
    # the coordinator step picks the shard; equals the single-call grouped draw with that group size
    B, D, V, shards = 7, 256, 128 * 24, 4
    per = V // shards
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=421)
    tau = np.linspace(0.7, 1.3, B).astype(np.float32)
    Hd, td = to_device_bf16(H), dev(tau, np.float32)
    for mode in (PAR, ONL):
        Ls, zs = [], []
        for r in range(shards):
            _, _, gl, gs = fs.flash_sample_grouped(Hd, to_device_bf16(W[r * per:(r + 1) * per]), td,
                                                   group_tiles=per // 128, mode=mode, seed=4,
                                                   vocab_offset=r * per, want_groups=True)
            assert gl.shape == (B, 1)
            Ls.append(gl)
            zs.append(gs)
        L = torch.cat(Ls, dim=1).contiguous()
        z = torch.cat(zs, dim=1).contiguous()
        c_i, c_l = fs.flash_group_choose(L, z, mode=mode, seed=4)
        w_i, w_l, wL, wz = fs.flash_sample_grouped(Hd, to_device_bf16(W), td, group_tiles=per // 128,
                                                   mode=mode, seed=4, want_groups=True)
        torch.cuda.synchronize()
        assert torch.equal(z, wz)
        assert torch.allclose(L, wL, rtol=0, atol=1e-5)
        assert torch.equal(c_i, w_i)
        assert torch.allclose(c_l, w_l, rtol=0, atol=1e-5)
        ref = orc.sample_grouped(H, W, tau, per, mode, seed=4)
        v = judge_grouped(orc, mode, ref, H, W, tau, c_i.cpu().numpy(), c_l.cpu().numpy(),
                          L.cpu().numpy(), z.cpu().numpy(), g=per, seed=4)
        assert v.ok, (mode, str(v), v.failures[:3])


@pytest.mark.parametrize("mode", [PAR, ONL])
def test_grouped_sampling_law_chi_square(fs, orc, mode):
    # many rows share one hidden vector; each row is an independent draw (row word differs)
    D, V, tau, n = 64, 640, 0.9, 30_000
    H1, W = wl.make_small(D=D, V=V, B=1, data_seed=422, w_row_scale=2.0)
    y = orc.logits(H1, W)[0]
    z = y / tau
    p = np.exp(z - z.max())
    p /= p.sum()
    Hd = to_device_bf16(np.repeat(H1, 500, axis=0))
    Wd = to_device_bf16(W)
    td = dev(np.full(500, tau), np.float32)
    counts = np.zeros(V, dtype=np.int64)
    for r in range(n // 500):
        idx, _, _, _ = fs.flash_sample_grouped(Hd, Wd, td, group_tiles=1, mode=mode, seed=77,
                                               row_offset=r * 500)
        counts += np.bincount(idx.cpu().numpy(), minlength=V)
    chi2, crit = _chi2_ok(counts, p, n)
    assert chi2 < crit, (mode, chi2, crit)


def test_grouped_at_llama_shape_sampled_rows(fs, orc):
    # full vocabulary width (1002 groups of one tile), reduced hidden size so the oracle finishes
    B, D, V = 6, 256, 128256
    print("grouped parity at V=128256", flush=True)
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=423)
    tau = np.array([0.5, 0.8, 1.0, 1.0, 1.3, 2.0], dtype=np.float32)
    for mode in (PAR, ONL):
        ref = orc.sample_grouped(H, W, tau, 128, mode, seed=6)
        gi, gl, gL, gz = run_grouped(fs, H, W, tau, 1, mode, seed=6)
        v = judge_grouped(orc, mode, ref, H, W, tau, gi, gl, gL, gz, g=128, seed=6)
        assert v.ok, (mode, str(v), v.failures[:3])
        for b in range(B):
            assert abs(gl[b] - ref["lse"][b]) <= lse_tol(tau[b], ref["lse"][b])
