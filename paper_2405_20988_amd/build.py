"""Compile the HIP library for gfx950, in-tree (paper_2405_20988_amd/lib/libfda.so).

The translation units are compiled in parallel and linked into one shared library."""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB_DIR = os.path.join(PKG, "lib")
OBJ_DIR = os.path.join(PKG, "_build")
LIB_PATH = os.path.join(LIB_DIR, "libfda.so")
EXAMPLE_SRC = os.path.join(CSRC, "fda_c_example.c")
EXAMPLE_PATH = os.path.join(LIB_DIR, "fda_c_example")
UNITS = (["fda_api", "fda_calibration"] +
         ["fda_state_narrow_%s_kc%d" % (t, k) for t in ("f32", "bf16") for k in (1, 2, 4, 6, 8)] +
         ["fda_state_wide_%s_%s" % (t, c) for t in ("f32", "bf16") for c in ("i64", "f64")] +
         ["fda_mean_%s_%s" % (t, c) for t in ("f32", "bf16") for c in ("i64", "f64")])
SOURCES = [os.path.join(CSRC, u + ".hip") for u in UNITS]
DEPENDS = SOURCES + [EXAMPLE_SRC] + [os.path.join(CSRC, n) for n in
                     ("fda_kernels.hpp", "fda_small_kernels.hpp", "fda_state_launch.hpp", "fda_state_narrow.inc",
                      "fda_state_wide.inc", "fda_mean_kernel.hpp", "fda_mean_launch.hpp", "fda_mean.inc")] + \
    [os.path.join(ROOT, "include", "fda.h")]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the FDA library needs the ROCm toolchain")
    return exe


def flags() -> list[str]:
    # FDA_EXTRA_HIPCC_FLAGS: extra compiler options, for experiments with the kernels' compile-time knobs
    extra = os.environ.get("FDA_EXTRA_HIPCC_FLAGS", "").split()
    return extra + ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
            # packed fp32 instructions are kept off for all device code
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + proc.stdout + proc.stderr)


def build_library(verbose: bool = False) -> str:
    """Always compiles; returns the path of the shared library."""
    os.makedirs(LIB_DIR, exist_ok=True)
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, u + ".o") for u in UNITS]
    cmds = [[hipcc()] + flags() + ["-c", src, "-o", obj] for src, obj in zip(SOURCES, objs)]
    # the units with the most worker slots take longest: start them first
    order = sorted(range(len(cmds)), key=lambda i: -int(UNITS[i].rsplit("kc", 1)[1]) if "kc" in UNITS[i] else 0)
    with ThreadPoolExecutor(max_workers=min(len(cmds), os.cpu_count() or 4)) as pool:
        list(pool.map(_run, [cmds[i] for i in order]))
    link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs
    _run(link)
    build_c_example()
    if verbose:
        for c in cmds + [link]:
            print(" ".join(c))
    return LIB_PATH


def build_c_example() -> str | None:
    """The plain C caller of the library (csrc/fda_c_example.c), built with the host C compiler
    against the HIP runtime; returns its path, or None without a C compiler."""
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        return None
    rocm = os.path.dirname(os.path.dirname(os.path.realpath(hipcc())))
    if not os.path.exists(os.path.join(rocm, "include", "hip", "hip_runtime_api.h")):
        rocm = "/opt/rocm"
    _run([cc, "-std=c99", "-O2", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
          "-I" + os.path.join(rocm, "include"), "-I" + os.path.join(ROOT, "include"), EXAMPLE_SRC,
          "-o", EXAMPLE_PATH, "-L" + LIB_DIR, "-lfda", "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
          "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")])
    return EXAMPLE_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in DEPENDS)


if __name__ == "__main__":
    print(build_library(verbose=False))
