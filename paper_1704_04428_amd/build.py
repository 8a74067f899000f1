"""Compile the HIP library for gfx950 into paper_1704_04428_amd/libconv_mcmk.so (in-tree)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "conv_mcmk.hip")
LIB = os.path.join(HERE, "libconv_mcmk.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    csrc = os.path.join(HERE, "csrc")
    inc = os.path.join(os.path.dirname(HERE), "include")
    out = [os.path.join(csrc, f) for f in sorted(os.listdir(csrc))]
    out += [os.path.join(inc, f) for f in sorted(os.listdir(inc))]
    return out


def is_current() -> bool:
    return os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in sources())


def build(force: bool = True, extra=()) -> str:
    if not force and os.path.exists(LIB):
        return LIB
    cmd = ["hipcc", *FLAGS, *extra, "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
