"""Compile the HIP library for gfx950 into ``paper_2507_10069_amd/libemm.so`` (in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libemm.so")
SOURCES = ["api.hip", "kv_scatter.hip", "attn_f32.hip", "attn_bf16.hip", "attn_bf16_decode.hip", "attn_merge.hip", "kv_migrate.hip", "prefix_cache.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instruction forms are switched off for every device translation unit
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# host-only translation units (no device code in them)
HOST_FLAGS = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-I", os.path.join(os.path.dirname(HERE), "include")]


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    flags = HOST_FLAGS if src.endswith(".cpp") else FLAGS + list(extra)
    cmd = [HIPCC] + flags + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    lines = [ln for ln in res.stderr.splitlines()
             if "packed-fp32-ops" not in ln and "is not a recognized feature" not in ln]
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr))
    if lines:
        sys.stderr.write("\n".join(lines) + "\n")
    return obj


def build(verbose: bool = False, extra_flags=()) -> str:
    """Always recompiles every translation unit, then links the shared library."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra_flags), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


TIMELINE_LIB = os.path.join(OBJ_DIR, "libemm_timeline.so")


def build_timeline(verbose: bool = False) -> str:
    """The library with the prefill kernel built with -DEMM_TIMELINE (every workgroup records when and where it ran
    at the head of the workspace); the other objects are those of the regular build.  For bench.py --timeline."""
    for src in SOURCES:
        if not os.path.exists(os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")):
            build()
            break
    obj = os.path.join(OBJ_DIR, "attn_bf16.timeline.o")
    res = subprocess.run([HIPCC] + FLAGS + ["-DEMM_TIMELINE", "-c", os.path.join(CSRC, "attn_bf16.hip"), "-o", obj],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for attn_bf16.hip (timeline):\n%s" % res.stderr)
    objs = [obj if s == "attn_bf16.hip" else os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", TIMELINE_LIB] + objs, check=True)
    if verbose:
        print("built", TIMELINE_LIB)
    return TIMELINE_LIB


SAN_LIB = os.path.join(OBJ_DIR, "libemm_san.so")
CLANG_RT_DIR = "/opt/rocm/lib/llvm/lib/clang"


def asan_runtime() -> str:
    """The shared AddressSanitizer runtime of the compiler hipcc drives (to be preloaded into a python process that
    loads the sanitized library)."""
    for root, _, files in os.walk(CLANG_RT_DIR):
        if "libclang_rt.asan-x86_64.so" in files:
            return os.path.join(root, "libclang_rt.asan-x86_64.so")
    raise FileNotFoundError("libclang_rt.asan-x86_64.so not found under " + CLANG_RT_DIR)


def build_sanitized(verbose: bool = False) -> str:
    """The same library with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (argument checks,
    planners, the prefix cache); device code is compiled as always.  Goes to _build/libemm_san.so; select it with
    EMM_LIB_PATH and preload asan_runtime().  Used by tests/test_sanitized_host.py, on the CPU."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    san_hip = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
               "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]
    san_cpp = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-fno-gpu-sanitize", "-g"]

    def one(src):
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".san.o")
        flags = [f for f in HOST_FLAGS if f != "-O3"] + ["-O1"] + san_cpp if src.endswith(".cpp") else FLAGS + san_hip
        res = subprocess.run([HIPCC] + flags + ["-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr))
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(one, SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-shared-libasan",
                    "-fno-gpu-sanitize", "-o", SAN_LIB] + objs, check=True, capture_output=True)
    if verbose:
        print("built", SAN_LIB)
    return SAN_LIB


if __name__ == "__main__":
    if sys.argv[1:] == ["--sanitize"]:
        build_sanitized(verbose=True)
    elif sys.argv[1:] == ["--timeline"]:
        build_timeline(verbose=True)
    else:
        build(verbose=True, extra_flags=sys.argv[1:])
