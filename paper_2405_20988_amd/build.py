"""Compile the HIP library for gfx950, in-tree (paper_2405_20988_amd/lib/libfda.so)."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB_DIR = os.path.join(PKG, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libfda.so")
SOURCES = [os.path.join(PKG, "csrc", "fda_api.hip")]
DEPENDS = SOURCES + [os.path.join(PKG, "csrc", "fda_kernels.hpp"),
                     os.path.join(ROOT, "include", "fda.h")]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the FDA library needs the ROCm toolchain")
    return exe


def command() -> list[str]:
    return [hipcc(), "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
            # packed fp32 instructions are kept off for all device code
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(PKG, "csrc"),
            "-o", LIB_PATH] + SOURCES


def build_library(verbose: bool = False) -> str:
    """Always compiles; returns the path of the shared library."""
    os.makedirs(LIB_DIR, exist_ok=True)
    cmd = command()
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + proc.stdout + proc.stderr)
    if verbose:
        print(" ".join(cmd))
    return LIB_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in DEPENDS)


if __name__ == "__main__":
    print(build_library(verbose=True))
