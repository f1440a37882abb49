"""Build the HIP library (libmpv.so) for gfx950, in-tree, with hipcc."""

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
SRC = os.path.join(PKG_DIR, "csrc", "mpv.hip")
LIB = os.path.join(PKG_DIR, "libmpv.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-shared",
    "-fPIC",
    # no compiler-generated packed-fp32 instructions (v_pk_*_f32)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the task loops are long and cold: loop-invariant constants hoisted out of them would be
    # held in registers across whole tasks and push the kept row pair into scratch memory
    "-mllvm", "-disable-machine-licm",
    "-Wno-unused-command-line-argument",
]


def hipcc_path():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build(verbose=True, extra_flags=()):
    """Compile csrc/mpv.hip into libmpv.so next to this file; always recompiles."""
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags,
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
           SRC, "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
