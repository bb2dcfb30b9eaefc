"""Compile the HIP sources into paper_2210_15748_amd/libdessert_hip.so for gfx950."""
from __future__ import annotations

import concurrent.futures
import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
CSRC = HERE / "csrc"
OBJ = HERE / "_build"
LIB = HERE / "libdessert_hip.so"
SOURCES = ["api.hip", "hash_kernels.hip", "score_kernels.hip", "topk_kernels.hip", "filter_kernels.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA accumulators in ordinary VGPRs: the sign packing reads them with VALU ops, which
         # cannot address AGPRs (saves one v_accvgpr_read per accumulator)
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         "-Wall", "-Wno-unused-command-line-argument"]


def stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    deps = list(CSRC.glob("*")) + [HERE.parent / "include" / "dessert.h"]
    return any(p.stat().st_mtime > t for p in deps)


def _compile(src: str, verbose: bool) -> pathlib.Path:
    obj = OBJ / (src.rsplit(".", 1)[0] + ".o")
    cmd = ["hipcc", *FLAGS, "-c", str(CSRC / src), "-o", str(obj)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return obj


def build(force: bool = True, verbose: bool = False) -> pathlib.Path:
    """One hipcc process per source file (the kernels do not call across files), then one link."""
    if not force and not stale():
        return LIB
    OBJ.mkdir(exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        objs = list(pool.map(lambda s: _compile(s, verbose), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *[str(o) for o in objs], "-o", str(LIB)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
