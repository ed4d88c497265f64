"""Build the HIP library (gfx950) in-tree: ``python -m paper_2603_15854_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libflashsample.so")
DEMO = os.path.join(HERE, "examples", "c_abi_demo")


def build(verbose: bool = False) -> str:
    """Compile csrc/flash_sample.hip for gfx950 into libflashsample.so (always recompiles)."""
    cmd = [
        "hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-command-line-argument",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        os.path.join(CSRC, "flash_sample.hip"), "-o", LIB,
    ]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 target feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed")
    if verbose and err.strip():
        sys.stderr.write(err + "\n")
    build_demo()
    return LIB


def build_demo() -> str:
    """Compile examples/c_abi_demo.c (plain C against the header) and link it with the library."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [
        "gcc", "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__",
        "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"),
        os.path.join(HERE, "examples", "c_abi_demo.c"),
        "-L", HERE, "-lflashsample", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
        "-Wl,-rpath,$ORIGIN/..", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", DEMO,
    ]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr + "\n")
        raise RuntimeError("building c_abi_demo failed")
    return DEMO


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
