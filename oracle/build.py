"""Compile the C oracle into ``oracle/_oracle.so`` with gcc.  Test infrastructure only."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle.c")
LIB = os.path.join(HERE, "_oracle.so")


def build(force: bool = False, src: str = SRC, lib: str = LIB) -> str:
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(src):
        return lib
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", lib, src, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True))
