"""Builds the C-ABI library `libhet_cache.so` for gfx950 with hipcc, in-tree.

    python -m paper_2112_07221_amd.build
"""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "het_cache.hip")
OUT = os.path.join(HERE, "libhet_cache.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # packed-fp32 instructions stay off: plain float code must not be fused into them
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def source_id() -> str:
    """Short hash of the sources the library is built from (the header and everything in csrc/):
    what `het_build_id()` returns, so that a measurement can name the build it was taken on."""
    h = hashlib.sha256()
    files = [os.path.join(HERE, "..", "include", "het_cache.h")]
    files += sorted(os.path.join(HERE, "csrc", f) for f in os.listdir(os.path.join(HERE, "csrc")))
    for f in files:
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:12]


def build(verbose: bool = False) -> str:
    cmd = [HIPCC, *FLAGS, f'-DHET_BUILD_ID="{source_id()}"', SRC, "-o", OUT]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
