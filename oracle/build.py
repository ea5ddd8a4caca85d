"""Compiles the CPU oracle (oracle/orc.c) into oracle/liborc.so with gcc.  Test infrastructure only."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liborc.so")
SRC = os.path.join(HERE, "orc.c")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-std=c99", "-O3", "-fopenmp", "-mavx2", "-mfma", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitize_check() -> str:
    """orc.c + sanitize_check.c as one executable under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).
    The sanitizer runtime is linked statically so that it does not depend on the order of preloaded libraries."""
    exe = os.path.join(HERE, "orc_sanitize_check")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-fopenmp", "-Wall", "-Wextra", "-o", exe,
           SRC, os.path.join(HERE, "sanitize_check.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    print(build())
