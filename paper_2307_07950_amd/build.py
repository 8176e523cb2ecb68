"""Build the HIP library in-tree for gfx950 with hipcc (no GPU needed)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libselsync.so")
SOURCES = ["selsync_host.hip", "selsync_kernels.hip", "selsync_noalloc.hip"]
HEADERS = ["selsync_internal.h", os.path.join("..", "..", "include", "selsync.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # one rounding per written fp32 operation: no multiply-add contraction anywhere
    "-ffp-contract=off",
    # IEEE-correct fp32 division and square root (the Adam variant relies on them)
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    # No packed-fp32 instructions (v_pk_add/mul/fma_f32) in device code.  The feature is taken by the
    # gfx950 device pass (tests/test_build_flags.py compiles a probe with and without it and reads the
    # emitted assembly); the x86 host pass does not know it and prints "not a recognized feature for
    # this target (ignoring feature)", which is harmless.
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not needs_build():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, "-o", tmp, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
