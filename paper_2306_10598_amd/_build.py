"""Builds libdc.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import subprocess
from pathlib import Path

HERE = Path(__file__).resolve().parent
ROOT = HERE.parent
LIB_PATH = HERE / "libdc.so"
SOURCES = [HERE / "csrc" / name for name in ("dc_api.hip", "dc_kernels.hip", "dc_rows.hip", "dc_rows_long.hip", "dc_row_lane.hip", "dc_trial.hip", "dc_workers.hip",
                                             "dc_analytic.hip")]
OBJECTS = HERE / "_build"                 # object files of the last build (git-ignored)

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def _compile(src: Path, verbose: bool) -> Path:
    obj = OBJECTS / (src.stem + ".o")
    cmd = ["hipcc", *HIPCC_FLAGS, f"-I{ROOT / 'include'}", f"-I{HERE / 'csrc'}", "-c", str(src), "-o", str(obj)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return obj


def build(verbose: bool = False) -> Path:
    """Compile every translation unit (side by side: the kernels with many instantiations take a minute each) and link."""
    from concurrent.futures import ThreadPoolExecutor
    OBJECTS.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        objects = list(pool.map(lambda src: _compile(src, verbose), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(LIB_PATH), *map(str, objects)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
