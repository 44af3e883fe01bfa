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
MICROBENCH_SRC = os.path.join(PKG, "csrc", "alu_issue_rates.hip")
MICROBENCH = os.path.join(PKG, "alu_issue_rates.bin")
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


STAMP = LIB + ".srchash"      # sha256 of the sources and flags the library beside it was built from


def source_hash(extra_flags=()) -> str:
    import hashlib
    h = hashlib.sha256()
    h.update("\0".join([*FLAGS, *extra_flags]).encode())
    for p in SOURCES + HEADERS + [EXAMPLE_SRC, MICROBENCH_SRC]:
        with open(p, "rb") as fh:
            h.update(b"\0" + os.path.basename(p).encode() + b"\0" + fh.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True if there is no library, or it was built from other sources than the ones in the tree (file
    times play no part: a copied tree keeps contents, not times)."""
    if not os.path.exists(LIB) or not os.path.exists(EXAMPLE) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as fh:
        return fh.read().strip() != source_hash()


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
    build_microbench()
    with open(STAMP, "w") as fh:
        fh.write(source_hash(extra_flags) + "\n")
    return LIB


def ensure_built() -> str:
    """What tests, the smoke run and the benchmark call: loads what is built, and builds (hipcc cross-compiles
    without a GPU) only if there is no library or the library was built from other sources than the tree holds,
    so that nothing is ever tested against a stale binary."""
    if is_stale():
        build()
    return LIB


def build_microbench() -> str:
    """The instruction-issue microbenchmark (a measurement aid, stand-alone, not linked to the library)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = MICROBENCH + f".tmp{os.getpid()}"
    res = subprocess.run([hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-o", tmp, MICROBENCH_SRC],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on the microbenchmark:\n" + res.stderr)
    os.replace(tmp, MICROBENCH)
    return MICROBENCH


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
