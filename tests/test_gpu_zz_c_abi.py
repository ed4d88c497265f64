"""The C ABI called from a plain C program (paper_2603_15854_amd/examples/c_abi_demo.c): same
inputs through the executable and through the oracle."""
import os
import subprocess

import numpy as np
import pytest

import fs_workloads as wl
from tests.parity import judge

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

DEMO = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                    "paper_2603_15854_amd", "examples", "c_abi_demo")


@pytest.mark.parametrize("shape", [(3, 512, 2000), (40, 256, 1500)])
def test_plain_c_program_matches_oracle(orc, tmp_path, shape):
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    assert os.path.exists(DEMO), "build the demo with `python -m paper_2603_15854_amd.build`"
    B, D, V = shape
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=660 + B)
    tau = np.linspace(0.7, 1.4, B).astype(np.float32)
    H.tofile(tmp_path / "h.bin")
    W.tofile(tmp_path / "w.bin")
    tau.tofile(tmp_path / "t.bin")
    out = tmp_path / "out.bin"
    res = subprocess.run([DEMO, str(tmp_path / "h.bin"), str(tmp_path / "w.bin"), str(tmp_path / "t.bin"),
                          str(B), str(D), str(V), "77", str(out)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, (res.stdout, res.stderr)
    raw = np.fromfile(out, dtype=np.uint8)
    idx = raw[:4 * B].view(np.int32)
    val = raw[4 * B:].view(np.float32)
    ref = orc.sample(H, W, tau, seed=77)
    v = judge(orc, H, W, tau, idx, val, ref, seed=77)
    assert v.ok, (shape, str(v), v.failures[:3], res.stdout)


def test_binding_loaded_before_torch_is_imported():
    # A process that loads the library first (build() followed by smoke() does) must end up with one HIP
    # runtime serving both the library and torch: the binding imports torch before it loads the library.
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2603_15854_amd as fs\n"
        "fs.lib()\n"
        "import torch, numpy as np\n"
        "import fs_workloads as wl\n"
        "from tests.parity import to_device_bf16\n"
        "H, W = wl.make_small(D=256, V=1000, B=4, data_seed=3)\n"
        "idx, val = fs.flash_sample_ex(to_device_bf16(H), to_device_bf16(W), torch.ones(4, device='cuda'), seed=5)\n"
        "torch.cuda.synchronize()\n"
        "print('IDX', idx.cpu().tolist())\n" % root)
    res = subprocess.run([os.sys.executable, "-c", code], capture_output=True, text=True, timeout=300, cwd=root)
    assert res.returncode == 0 and "IDX" in res.stdout, (res.stdout[-500:], res.stderr[-1500:])
