"""Compile the HIP attention library for gfx950 into paper_2410_20399_amd/libtk_attn.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtk_attn.so")
SOURCES = ["tk_attn_api.hip", "attn_fwd.hip", "attn_bwd.hip", "mfma_probe.hip", "rotary.hip", "gemm.hip"]
HEADERS = ["tk_common.h", "tk_launch.h", os.path.join("..", "..", "include", "tk_attn.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept off for every HIP translation unit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True, extra_flags=()) -> str:
    if not force and not stale():
        return LIB
    cmd = ["hipcc", *FLAGS, *extra_flags, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
