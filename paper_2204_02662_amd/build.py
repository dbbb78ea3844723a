"""Build libepp.so (HIP, gfx950) in-tree."""
from __future__ import annotations

import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
SO = PKG / "libepp.so"
SOURCES = sorted((PKG / "csrc").glob("*.hip"))

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False) -> Path:
    cmd = ["hipcc", *HIPCC_FLAGS, f"-I{ROOT / 'include'}", f"-I{PKG / 'csrc'}",
           *map(str, SOURCES), "-o", str(SO)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return SO


if __name__ == "__main__":
    build(verbose=True)
