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
    # schedule for instruction-level parallelism: the event loops are issue- and
    # latency-bound at two or three wavefronts per SIMD (one for the traces), and
    # the default, which schedules for occupancy, leaves 2-4 % on the table
    # (measured on every bench workload; the planner alone loses 3 %)
    "-mllvm", "-amdgpu-sched-strategy=max-ilp",
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


def exec_hazards(asm_text: str):
    """The event loops switch the active lanes inside inline-assembly blocks
    (v_cmpx ... s_mov exec), into which the compiler's hazard recogniser does
    not look.  On this target an instruction that reads other lanes (DPP,
    v_readlane, v_readfirstlane, v_writelane, v_permlane) needs up to five wait
    states after a vector instruction that wrote exec.  Returns the blocks
    after whose last v_cmpx fewer instructions than that come before such an
    instruction, as (instructions inside the block after it, the window)."""
    import re
    lines = asm_text.split("\n")
    found, blocks, i = [], 0, 0
    while i < len(lines):
        if "ASMSTART" in lines[i]:
            j = i
            while "ASMEND" not in lines[j]:
                j += 1
            block = [l.strip() for l in lines[i + 1:j] if l.strip() and not l.strip().startswith(";")]
            if any(l.startswith("v_cmpx") for l in block):
                blocks += 1
                last = max(k for k, l in enumerate(block) if l.startswith("v_cmpx"))
                inside = len(block) - last - 1
                follow, k = [], j + 1
                while len(follow) < 5 and k < len(lines):
                    l = lines[k].strip()
                    k += 1
                    if l and l[0] not in ";." and not l.endswith(":"):
                        follow.append(l)
                window = follow[:max(0, 5 - inside)]
                if any(re.search(r"dpp|readlane|readfirstlane|writelane|permlane", l) for l in window):
                    found.append((inside, window))
            i = j
        i += 1
    return blocks, found


def device_assembly() -> str:
    """The device code of the library as assembly text (same flags as build())."""
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [HIPCC, *flags, "-S", "--cuda-device-only", "-o", "-", *SOURCES]
    return subprocess.run(cmd, check=True, capture_output=True, text=True).stdout


def ensure_built() -> str:
    """Build only if no library is there at all (tests, smoke and bench call
    this; the binding itself never builds and fails loudly instead)."""
    return LIB if os.path.exists(LIB) else build(force=True)


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
