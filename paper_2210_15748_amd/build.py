"""Compile the HIP sources into paper_2210_15748_amd/libdessert_hip.so for gfx950."""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libdessert_hip.so"
SOURCES = ["api.hip", "hash_kernels.hip", "score_kernels.hip", "topk_kernels.hip", "filter_kernels.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
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


def build(force: bool = True, verbose: bool = False) -> pathlib.Path:
    if not force and not stale():
        return LIB
    cmd = ["hipcc", *FLAGS, *[str(CSRC / s) for s in SOURCES], "-o", str(LIB)]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
