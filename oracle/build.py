"""Compile the CPU checker (plain C, gcc) into oracle/libgf_oracle.so."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gf_oracle.c")
LIB = os.path.join(HERE, "libgf_oracle.so")
LIB_SANITIZED = os.path.join(HERE, "libgf_oracle_asan.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized() -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).  A
    process that loads it must have the ASan runtime loaded first (LD_PRELOAD of gcc's libasan.so)."""
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB_SANITIZED, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB_SANITIZED


if __name__ == "__main__":
    print(build(force=True))
