"""Build libepp.so (HIP, gfx950) in-tree."""
from __future__ import annotations

import hashlib
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


STAMP = PKG / "libepp.so.sources"  # hash of the sources the library file was built from


def source_hash() -> str:
    """Hash of everything under csrc/ (names and contents)."""
    h = hashlib.sha256()
    for f in sorted((PKG / "csrc").glob("*")):
        h.update(f.name.encode())
        h.update(f.read_bytes())
    return h.hexdigest()[:16]


def build(verbose: bool = False) -> Path:
    cmd = ["hipcc", *HIPCC_FLAGS, f"-I{ROOT / 'include'}", f"-I{PKG / 'csrc'}",
           *map(str, SOURCES), "-o", str(SO)]
    if verbose:
        print(" ".join(cmd), flush=True)
    stamp = source_hash()
    STAMP.unlink(missing_ok=True)
    subprocess.check_call(cmd)
    STAMP.write_text(stamp + "\n")  # (a library left over from other sources is then recognisable)
    return SO


if __name__ == "__main__":
    build(verbose=True)
