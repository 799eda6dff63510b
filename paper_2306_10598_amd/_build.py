"""Builds libdc.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import subprocess
from pathlib import Path

HERE = Path(__file__).resolve().parent
ROOT = HERE.parent
LIB_PATH = HERE / "libdc.so"
SOURCES = [HERE / "csrc" / "dc_api.hip", HERE / "csrc" / "dc_kernels.hip", HERE / "csrc" / "dc_analytic.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def build(verbose: bool = False) -> Path:
    cmd = ["hipcc", *HIPCC_FLAGS, f"-I{ROOT / 'include'}", f"-I{HERE / 'csrc'}",
           "-o", str(LIB_PATH), *map(str, SOURCES)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
