"""Compile the C oracle into oracle/libconv_oracle.so with gcc (host only, no HIP).

TEST INFRASTRUCTURE ONLY: see conv_oracle.c.

    python -m oracle.build             the library the tests load
    python -m oracle.build --sanitize  oracle/conv_oracle_asan: the hand-worked pins compiled into a host program
                                       with -fsanitize=address,undefined (see sanitize_check.c)
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "conv_oracle.c")
HDR = os.path.join(HERE, "conv_oracle.h")
LIB = os.path.join(HERE, "libconv_oracle.so")
CHECK_SRC = os.path.join(HERE, "sanitize_check.c")
CHECK_BIN = os.path.join(HERE, "conv_oracle_asan")


def build(force: bool = True) -> str:
    newest = max(os.path.getmtime(SRC), os.path.getmtime(HDR))
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= newest:
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized() -> str:
    """The oracle and a small driver (sanitize_check.c) as one host program under AddressSanitizer and
    UndefinedBehaviorSanitizer, single-threaded so that every report is deterministic."""
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-Wno-unknown-pragmas", "-o", CHECK_BIN, CHECK_SRC, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return CHECK_BIN


if __name__ == "__main__":
    print(build_sanitized() if "--sanitize" in sys.argv[1:] else build())
