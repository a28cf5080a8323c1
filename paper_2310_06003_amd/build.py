"""Builds libparo.so (host plan + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

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


def stale() -> bool:
    if not os.path.exists(SO):
        return True
    t = os.path.getmtime(SO)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + SOURCES + ["-o", SO]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return SO


if __name__ == "__main__":
    build(verbose=True)
