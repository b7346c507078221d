"""Build ``libnormtest.so`` from ``csrc/normtest.hip`` for gfx950 with hipcc (works without a GPU)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SRC = os.path.join(_HERE, "csrc", "normtest.hip")
LIB = os.path.join(_HERE, "libnormtest.so")
INCLUDE = os.path.join(ROOT, "include")

# contraction off: the error-free transformations of the finalize kernel and the bit-identical
# fast/guarded paths rely on every fused multiply-add being an explicit one;
# packed fp32 instructions are disabled for the device pass.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(out: str = LIB, quiet: bool = True) -> str:
    cmd = ["hipcc", *HIPCC_FLAGS, "-I", INCLUDE]
    tmp = out + ".tmp.%d" % os.getpid()
    cmd += ["-o", tmp, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n%s\n%s" % (" ".join(cmd), res.stderr))
    if not quiet:
        # the host pass does not know the device-only target feature and says so: harmless
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    os.replace(tmp, out)
    return out


def ensure_built() -> str:
    """Path of the built library; builds it if nothing is there or a source is newer than the build."""
    header = os.path.join(INCLUDE, "normtest.h")
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(SRC), os.path.getmtime(header)):
        build_library()
    return LIB


if __name__ == "__main__":
    print(build_library(quiet=False))
