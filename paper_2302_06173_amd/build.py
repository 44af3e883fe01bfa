"""Build the HIP library in-tree: csrc/api.hip -> libswift_undo.so (gfx950 only).

Run as ``python -m paper_2302_06173_amd.build``; ``__graft_entry__.build()`` calls ``build()``.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libswift_undo.so")
SOURCES = [os.path.join(PKG, "csrc", "api.hip")]
HEADERS = [os.path.join(PKG, "csrc", h) for h in
           ("opt_kernels.hpp", "digest_kernels.hpp", "lamb_kernels.hpp", "fused_kernels.hpp", "logging_groups.hpp")] + \
          [os.path.join(ROOT, "include", "swift_undo.h")]
EXAMPLE_SRC = os.path.join(PKG, "csrc", "example_undo_roundtrip.c")
EXAMPLE = os.path.join(PKG, "example_undo_roundtrip.bin")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # explicit FMAs only: the vector body and the scalar head/tail must round identically
    "-ffp-contract=off",
    # no compiler-generated packed-fp32 instructions on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra",
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS + [EXAMPLE_SRC]) or not os.path.exists(EXAMPLE)


def build(force: bool = True, extra_flags=()) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc, *FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
           "-o", tmp, *SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    if err.strip():
        print(err, file=sys.stderr)
    os.replace(tmp, LIB)
    build_example()
    return LIB


def ensure_built() -> str:
    """Build only if no library is there (tests, the smoke run and the benchmark call this; they never
    rebuild what exists, so build again yourself after changing a source)."""
    if not os.path.exists(LIB):
        build()
    elif not os.path.exists(EXAMPLE):
        build_example()
    return LIB


def build_example() -> str:
    """The plain-C example program: gcc, linked against the library and the HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    tmp = EXAMPLE + f".tmp{os.getpid()}"
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(ROOT, "include"), EXAMPLE_SRC, "-L", PKG, "-lswift_undo", "-L", os.path.join(rocm, "lib"),
           "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + " ".join(cmd) + "\n" + res.stderr)
    os.replace(tmp, EXAMPLE)
    return EXAMPLE


if __name__ == "__main__":
    print(build())
