"""GPU parity of flash_sample_full (additive bias, allowed-id mask, log-normaliser) against the
oracle's fso_sample_full on the same seeded inputs."""
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


def dev_words(words):
    return None if words is None else torch.from_numpy(np.ascontiguousarray(words).view(np.int32)).cuda()


def run_full(fs, H, W, tau, *, seed=0, row_seeds=None, bias=None, words=None, Wd=None, **kw):
    idx, val, lse = fs.flash_sample_full(to_device_bf16(H), to_device_bf16(W) if Wd is None else Wd,
                                         dev(tau, np.float32), seed=seed, row_seeds=to_device_seeds(row_seeds),
                                         bias=None if bias is None else dev(bias, np.float32),
                                         allowed=dev_words(words), **kw)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), val.cpu().numpy(), lse.cpu().numpy()


def lse_tol(tau, lse):
    return 2e-3 / min(float(tau), 1.0) + 1e-5 * abs(float(lse)) + 1e-4


CASES = [
    # (B, D, V): split-K kernel (B <= 16), tiled kernels with 32 / 64 / 128-row batch tiles, ragged edges
    (5, 512, 1189), (16, 4096, 2048 + 64), (1, 256, 4096), (9, 7168, 520), (3, 24, 127), (2, 8, 5),
    (40, 1032, 1300), (64, 512, 700), (100, 264, 640), (130, 2048, 515), (300, 256, 1000),
]


@pytest.mark.parametrize("shape", CASES)
@pytest.mark.parametrize("mode", ["bias+rowmask", "sharedmask", "bias", "plain"])
def test_full_transform_matches_oracle(fs, orc, shape, mode):
    B, D, V = shape
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=300 + B + V)
    rng = np.random.default_rng(B * 7 + V)
    tau = np.linspace(0.6, 1.6, B).astype(np.float32)
    bias = rng.normal(0, 1.0, V).astype(np.float32) if "bias" in mode else None
    words = None
    if mode == "bias+rowmask":
        allowed = rng.random((B, V)) < 0.6
        allowed[:, V // 2] = True
        words = orc.pack_allowed(allowed)
    elif mode == "sharedmask":
        allowed = rng.random(V) < 0.5
        allowed[0] = True
        words = orc.pack_allowed(allowed)
    ref = orc.sample_full(H, W, tau, seed=31, bias=bias, allowed_words=words)
    gi, gv, gl = run_full(fs, H, W, tau, seed=31, bias=bias, words=words)
    v = judge(orc, H, W, tau, gi, gv, ref, seed=31, bias=bias, allowed_words=words)
    assert v.ok, (shape, mode, str(v), v.failures[:3])
    for b in range(B):
        assert abs(gl[b] - ref["lse"][b]) <= lse_tol(tau[b], ref["lse"][b]), (shape, mode, b, gl[b], ref["lse"][b])
    if words is not None:     # a masked id is never returned
        for b in range(B):
            row = words if words.ndim == 1 else words[b]
            assert (row[gi[b] >> 5] >> (gi[b] & 31)) & 1


def test_full_without_transform_equals_plain_entry(fs, orc):
    H, W = wl.make_small(D=1024, V=3000, B=24, data_seed=310)
    tau = np.full(24, 0.9, dtype=np.float32)
    Hd, Wd, td = to_device_bf16(H), to_device_bf16(W), dev(tau, np.float32)
    a_i, a_v = fs.flash_sample_ex(Hd, Wd, td, seed=5)
    b_i, b_v, b_l = fs.flash_sample_full(Hd, Wd, td, seed=5)
    c_i, c_v, c_l = fs.flash_sample_full(Hd, Wd, td, seed=5, want_lse=False)
    torch.cuda.synchronize()
    assert torch.equal(a_i, b_i) and torch.equal(a_i, c_i) and c_l is None
    assert torch.allclose(a_v, b_v, rtol=0, atol=2e-6 * 16)
    Y = orc.logits(H, W)
    for b in range(24):
        assert abs(float(b_l[b]) - orc.log_sum_exp(Y[b] / 0.9)) <= lse_tol(0.9, 10.0)


def test_rows_with_everything_masked_and_single_allowed_id(fs, orc):
    B, D, V = 20, 256, 900
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=311)
    tau = np.ones(B, dtype=np.float32)
    allowed = np.ones((B, V), dtype=bool)
    allowed[3, :] = False                      # nothing allowed
    allowed[7, :] = False
    allowed[7, 555] = True                     # exactly one id allowed
    allowed[19, :] = False
    allowed[19, V - 1] = True                  # the last id, in the ragged last tile
    words = orc.pack_allowed(allowed)
    gi, gv, gl = run_full(fs, H, W, tau, seed=2, words=words)
    assert gi[3] == -1 and gv[3] == -np.inf and gl[3] == -np.inf
    assert gi[7] == 555 and gi[19] == V - 1
    Y = orc.logits(H, W)
    assert abs(gl[7] - Y[7, 555]) <= 2e-3 and abs(gl[19] - Y[19, V - 1]) <= 2e-3
    ref = orc.sample_full(H, W, tau, seed=2, allowed_words=words)
    assert np.array_equal(ref["idx"], gi)


def test_masked_sampling_law_chi_square(fs, orc):
    from scipy import stats
    D, V, tau, n = 64, 512, 0.9, 30_000
    H1, W = wl.make_small(D=D, V=V, B=1, data_seed=312, w_row_scale=2.0)
    rng = np.random.default_rng(4)
    bias = rng.normal(0, 1, V).astype(np.float32)
    allowed = rng.random(V) < 0.5
    words = orc.pack_allowed(allowed)
    z = (orc.logits(H1, W)[0] + bias) / tau
    p = np.where(allowed, np.exp(z - z[allowed].max()), 0.0)
    p /= p.sum()
    gi, _, gl = run_full(fs, np.repeat(H1, n, axis=0), W, np.full(n, tau, np.float32), seed=99, bias=bias, words=words)
    counts = np.bincount(gi, minlength=V)
    assert counts[~allowed].sum() == 0
    order = np.argsort(p[allowed])
    e, c = (p[allowed] * n)[order], counts[allowed][order]
    ce, cc, E, C = 0.0, 0, [], []
    for ei, ci in zip(e, c):
        ce += ei; cc += ci
        if ce >= 5:
            E.append(ce); C.append(cc); ce, cc = 0.0, 0
    E[-1] += ce; C[-1] += cc
    E, C = np.array(E), np.array(C)
    assert ((C - E) ** 2 / E).sum() < stats.chi2.ppf(0.999, len(E) - 1)
    assert np.all(np.abs(gl - orc.log_sum_exp(np.where(allowed, z, -np.inf))) <= lse_tol(tau, 10.0))


def test_full_transform_at_llama_shape(fs, orc):
    w = wl.WORKLOADS["C2"]
    Wb = wl.make_weights(w)
    Wd = to_device_bf16(Wb)
    rng = np.random.default_rng(12)
    bias = rng.normal(0, 0.5, w.V).astype(np.float32)
    for B in (16, 64):
        H = wl.make_hidden(w, B)
        tau = np.linspace(0.7, 1.3, B).astype(np.float32)
        allowed = rng.random((B, w.V)) < 0.7
        words = orc.pack_allowed(allowed)
        gi, gv, gl = run_full(fs, H, Wb, tau, seed=1, bias=bias, words=words, Wd=Wd)
        ref = orc.sample_full(H, Wb, tau, seed=1, bias=bias, allowed_words=words)
        v = judge(orc, H, Wb, tau, gi, gv, ref, seed=1, bias=bias, allowed_words=words)   # every row
        print(f"[parity] full transform C2 B={B} all rows: {v}", flush=True)
        assert v.rows == B and v.ok, (B, str(v), v.failures[:3])
        for b in range(B):
            assert allowed[b, gi[b]]
            assert abs(gl[b] - ref["lse"][b]) <= lse_tol(tau[b], ref["lse"][b])


def test_full_entry_rejects_bad_arguments(fs):
    H = torch.zeros((4, 256), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((300, 256), dtype=torch.bfloat16, device="cuda")
    tau = torch.ones(4, device="cuda")
    short = torch.zeros((4, 5), dtype=torch.int32, device="cuda")     # needs ceil(300/32) = 10 words per row
    with pytest.raises(ValueError):                 # the binding sees the short rows first
        fs.flash_sample_full(H, W, tau, allowed=short)
    ws = torch.empty(fs.flash_sample_full_workspace_bytes(4, 300), dtype=torch.uint8, device="cuda")
    oi = torch.empty(4, dtype=torch.int32, device="cuda")
    ov = torch.empty(4, dtype=torch.float32, device="cuda")
    st = fs.lib().flash_sample_full(H.data_ptr(), W.data_ptr(), 4, 256, 300, tau.data_ptr(), 0, None, 0, 0, None,
                                    short.data_ptr(), 5, oi.data_ptr(), ov.data_ptr(), None, ws.data_ptr(),
                                    ws.numel(), None, 0)
    assert st == fs.FS_ERR_SHAPE                    # and so does the library itself
    with pytest.raises(fs.FlashSampleError) as e:
        fs.flash_sample_full(H, W, tau, flags=fs.FS_VARIANT(3))
    assert e.value.status == fs.FS_ERR_UNSUPPORTED
    with pytest.raises(fs.FlashSampleError) as e:
        fs.flash_sample_full(H, W, tau, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == fs.FS_ERR_WORKSPACE


@pytest.mark.parametrize("B", [24, 48, 80, 140])
def test_full_transform_at_full_vocabulary_width(fs, orc, B):
    # V = 128256 makes the launcher pick its one-workgroup-per-CU tile shapes (256 and 512 rows);
    # the hidden size is kept small so that the oracle finishes in seconds
    D, V = 128, 128256
    print(f"full transform, V={V}, B={B}", flush=True)
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=330 + B)
    rng = np.random.default_rng(B)
    tau = np.linspace(0.7, 1.4, B).astype(np.float32)
    bias = rng.normal(0, 1.0, V).astype(np.float32)
    allowed = rng.random(V) < 0.6
    allowed[V - 1] = True
    words = orc.pack_allowed(allowed)
    ref = orc.sample_full(H, W, tau, seed=8, bias=bias, allowed_words=words)
    gi, gv, gl = run_full(fs, H, W, tau, seed=8, bias=bias, words=words)
    v = judge(orc, H, W, tau, gi, gv, ref, seed=8, bias=bias, allowed_words=words)
    assert v.ok, (B, str(v), v.failures[:3])
    for b in range(B):
        assert abs(gl[b] - ref["lse"][b]) <= lse_tol(tau[b], ref["lse"][b])
