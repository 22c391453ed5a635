"""Builds libkeyformer.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkeyformer.so")
SOURCES = ["kf_api.hip", "kf_decode.hip", "kf_select.hip", "kf_prefill.hip"]
HEADERS = ["kf_device.h", "kf_internal.h", "kf_merge.h", os.path.join("..", "..", "include", "keyformer.h")]
EXAMPLE_SRC = os.path.join(HERE, "examples", "generate_loop.cpp")
EXAMPLE_BIN = os.path.join(HERE, "examples", "generate_loop")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        compile_flags = [f for f in FLAGS if f != "-shared"]
        objdir = os.path.join(HERE, "_build")
        os.makedirs(objdir, exist_ok=True)

        def compile_one(src):
            obj = os.path.join(objdir, src.replace(".hip", ".o"))
            cmd = [hipcc] + compile_flags + ["-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
            return obj

        # one compiler process per source file, side by side
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    build_example(force, verbose)
    return LIB


def build_example(force: bool = True, verbose: bool = False) -> str:
    """The stand-alone C++ user of the C ABI (no Python, no torch), linked against the in-tree library."""
    if force or not os.path.exists(EXAMPLE_BIN) or os.path.getmtime(EXAMPLE_BIN) < max(
            os.path.getmtime(EXAMPLE_SRC), os.path.getmtime(LIB)):
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wall", "-Wextra", EXAMPLE_SRC,
               "-I", os.path.join(HERE, "..", "include"), "-L", HERE, "-lkeyformer", "-Wl,-rpath,$ORIGIN/..",
               "-o", EXAMPLE_BIN]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
