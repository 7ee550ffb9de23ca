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


def build_sanitized(lib: str = os.path.join(HERE, "_oracle_san.so"), src: str = SRC) -> str:
    """The oracle under AddressSanitizer and UndefinedBehaviorSanitizer, with the clang that ships with ROCm (so that
    it shares one sanitizer runtime with the sanitized HIP library in a process that loads both) and without OpenMP."""
    clang = "/opt/rocm/lib/llvm/bin/clang"
    cmd = [clang, "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-Wno-unknown-pragmas", "-Wno-source-uses-openmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared-libasan", "-o", lib, src, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True))
