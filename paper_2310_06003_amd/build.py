"""Builds libparo.so (host plan + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SO = os.path.join(HERE, "libparo.so")
SOURCES = [os.path.join(HERE, "csrc", "plan.cpp"), os.path.join(HERE, "csrc", "kernels.hip")]
HEADERS = [os.path.join(HERE, "csrc", h) for h in ("plan.hpp", "device_util.hpp", "loaders.hpp")] + \
          [os.path.join(ROOT, "include", "paro.h")]

# -ffp-contract=off: every fp32 operation of the fold and of Adam is rounded on its own, so
#   results do not depend on which multiply-adds the compiler could fuse.
# -packed-fp32-ops off: scalar fp32 arithmetic only.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
         "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]


STAMP = SO + ".srchash"        # hash of what the library in the tree was built from


def source_hash() -> str:
    """sha256 over the compiler flags and the text of every source and header."""
    h = hashlib.sha256(" ".join(FLAGS[:-2]).encode())          # without the two -I paths (they differ per checkout)
    for f in SOURCES + HEADERS:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def built_hash() -> str:
    """The source hash recorded when the library in the tree was built ("" if unknown)."""
    try:
        with open(STAMP) as fh:
            return fh.read().strip()
    except OSError:
        return ""


def stale() -> bool:
    """True when there is no library, or it was built from other sources than the tree holds."""
    return not os.path.exists(SO) or built_hash() != source_hash()


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + SOURCES + ["-o", SO]
    if verbose:
        print(" ".join(cmd))
    if os.path.exists(STAMP):
        os.remove(STAMP)
    subprocess.run(cmd, check=True)
    with open(STAMP, "w") as fh:
        fh.write(source_hash() + "\n")
    return SO


if __name__ == "__main__":
    build(verbose=True)
