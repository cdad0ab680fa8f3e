"""Build step: compiles the HIP sources for gfx950 into libcats.so (in-tree)."""
from __future__ import annotations

import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
LIB = PKG / "libcats.so"
SOURCES = ["gemm.hip", "gemv.hip", "rowops.hip", "attention.hip", "accept.hip", "loss.hip", "api.hip"]


def build_library(verbose: bool = False) -> Path:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           f"-I{ROOT / 'include'}", f"-I{PKG / 'csrc'}"]
    cmd += [str(PKG / "csrc" / s) for s in SOURCES]
    cmd += ["-o", str(LIB)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
