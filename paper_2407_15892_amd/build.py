"""Builds libmst_lmhead.so and libmst_mlp.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libmst_lmhead.so")
MLP_LIB_PATH = os.path.join(HERE, "libmst_mlp.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def find_hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; a ROCm toolchain is required to build the library")


def _compile(src_name: str, lib_path: str, verbose: bool) -> str:
    src = os.path.join(CSRC, src_name)
    tmp = lib_path + ".tmp"
    cmd = [find_hipcc(), *HIPCC_FLAGS, "-o", tmp, src]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr[-4000:])
    os.replace(tmp, lib_path)
    return lib_path


def build(verbose: bool = False) -> str:
    """Compile csrc/mst_api.hip into libmst_lmhead.so and csrc/mst_mlp_api.hip into libmst_mlp.so;
    returns the path of the LM-head library."""
    _compile("mst_mlp_api.hip", MLP_LIB_PATH, verbose)
    return _compile("mst_api.hip", LIB_PATH, verbose)


if __name__ == "__main__":
    print(build(verbose=True))
