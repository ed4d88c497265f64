"""Build the HIP library (gfx950) in-tree: ``python -m paper_2603_15854_amd.build [-v]``.

Each kernel family is its own translation unit (``csrc/*.hip``); the units are compiled in
parallel into ``_build/*.o`` and linked into ``libflashsample.so`` next to this file.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflashsample.so")
DEMO = os.path.join(HERE, "examples", "c_abi_demo")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _filter(stderr: str) -> str:
    # the host pass warns that it does not know the packed-fp32 target feature: harmless
    return "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l)


def _compile(src: str, verbose: bool) -> str:
    obj = os.path.join(OBJ, os.path.splitext(os.path.basename(src))[0] + ".o")
    cmd = ["hipcc", *HIPCC_FLAGS, "-c", src, "-o", obj]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = _filter(res.stderr)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError(f"hipcc failed on {os.path.basename(src)}")
    if verbose and err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compile every csrc/*.hip for gfx950 and link libflashsample.so (always recompiles)."""
    os.makedirs(OBJ, exist_ok=True)
    sources = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(sources)))) as ex:
        objs = list(ex.map(lambda s: _compile(s, verbose), sources))
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                         capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(_filter(res.stderr) + "\n")
        raise RuntimeError("linking libflashsample.so failed")
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
