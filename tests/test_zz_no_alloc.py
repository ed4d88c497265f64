"""flash_sample_static -- the entry point that allocates nothing (its candidate buffer is a device
array built into the library) -- against flash_sample_ex on the same inputs, through the C ABI.
Two calls in a row, the second on a smaller problem: the scratch keeps the first call's contents,
and the second result must not see them.  Runs last (file name) and also alone in a fresh process."""
import numpy as np
import pytest

import fs_workloads as wl
from tests.parity import judge, to_device_bf16

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def fs():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    import paper_2603_15854_amd as fs
    fs.lib()
    return fs


def _case(fs, orc, B, D, V, data_seed, seed, check_oracle):
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=data_seed)
    Hd, Wd = to_device_bf16(H), to_device_bf16(W)
    tau_h = np.linspace(0.7, 1.3, B).astype(np.float32)
    tau = torch.from_numpy(tau_h).cuda()
    seeds_h = (np.arange(B, dtype=np.uint64) * np.uint64(3) + np.uint64(1))
    seeds = torch.from_numpy(seeds_h.view(np.int64)).cuda()
    oi = torch.full((B,), -5, dtype=torch.int32, device="cuda")
    ov = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
    fs.flash_sample_static(Hd, Wd, tau, oi, ov, seed=seed, row_seeds=seeds, row_offset=7, vocab_offset=128)
    torch.cuda.synchronize()
    ei, ev = fs.flash_sample_ex(Hd, Wd, tau, seed=seed, row_seeds=seeds, row_offset=7, vocab_offset=128)
    torch.cuda.synchronize()
    # integer output bit-exact; the value is the same kernel on the same inputs, hence bit-exact too
    assert torch.equal(oi, ei), (B, D, V)
    assert torch.equal(ov, ev), (B, D, V)
    if check_oracle:
        ref = orc.sample(H, W, tau_h, seed=seed, row_seeds=seeds_h, row_offset=7, vocab_offset=128)
        v = judge(orc, H, W, tau_h, oi.cpu().numpy(), ov.cpu().numpy(), ref, seed=seed, row_seeds=seeds_h,
                  row_offset=7, vocab_offset=128)
        assert v.ok, (B, D, V, str(v), v.failures[:3])


def test_static_scratch_entry_point_matches_workspace_entry_point(fs, orc):
    # first call: several batch tiles and a ragged last vocabulary tile (tiled kernel); second call:
    # fewer rows and fewer tiles (split-K kernel), so most of the scratch still holds the first call's candidates
    print("flash_sample_static: B=200 D=512 V=128*37+5", flush=True)
    _case(fs, orc, 200, 512, 128 * 37 + 5, data_seed=901, seed=11, check_oracle=True)
    print("flash_sample_static: B=5 D=1024 V=128*9+1", flush=True)
    _case(fs, orc, 5, 1024, 128 * 9 + 1, data_seed=902, seed=12, check_oracle=True)
    # and once more at the first size: the result does not depend on what the scratch held
    _case(fs, orc, 200, 512, 128 * 37 + 5, data_seed=901, seed=11, check_oracle=False)


def test_static_scratch_limit_is_an_error_not_a_fault(fs):
    V = 128 * 1200
    B = fs.FS_STATIC_SCRATCH_BYTES // (8 * 1200) + 1
    assert fs.flash_sample_workspace_bytes(B, V) > fs.FS_STATIC_SCRATCH_BYTES
    H = torch.zeros((B, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((V, 64), dtype=torch.bfloat16, device="cuda")
    tau = torch.ones(B, device="cuda")
    oi = torch.empty(B, dtype=torch.int32, device="cuda")
    ov = torch.empty(B, dtype=torch.float32, device="cuda")
    with pytest.raises(fs.FlashSampleError) as e:
        fs.flash_sample_static(H, W, tau, oi, ov)
    assert e.value.status == fs.FS_ERR_SCRATCH_LIMIT
