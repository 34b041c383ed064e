"""Compile the HIP kernels and their C ABI for gfx950 into
paper_2110_04478_amd/libthemis_hip.so (cross-compiles without a GPU)."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
PKG = os.path.dirname(HERE)
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libthemis_hip.so")
SOURCES = [os.path.join(HERE, "themis_api.hip")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # every product and sum rounds once, in source order (bit-exact parity)
    "-ffp-contract=off", "-fno-fast-math",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", HERE,
    "-Wall", "-Wno-unused-function",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    deps = glob.glob(os.path.join(HERE, "*.h*")) + [os.path.join(ROOT, "include", "themis.h")]
    return any(os.path.getmtime(d) > os.path.getmtime(LIB) for d in deps)


def build(force: bool = True, extra=()) -> str:
    if not force and not stale():
        return LIB
    cmd = [HIPCC, *FLAGS, *extra, "-o", LIB, *SOURCES]
    subprocess.run(cmd, check=True)
    return LIB


def ensure_built() -> str:
    """Build only if no library is there at all (tests, smoke and bench call
    this; the binding itself never builds and fails loudly instead)."""
    return LIB if os.path.exists(LIB) else build(force=True)


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
