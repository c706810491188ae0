"""Build the HIP library in-tree: ``python -m paper_2605_00392_amd.build``.

hipcc cross-compiles for gfx950 without a GPU.  The shared object lands next to
this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "librtprune.so")
SOURCES = [os.path.join(HERE, "csrc", "rtprune.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# packed fp32 instructions are switched off for all device code on purpose
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
]


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile ``csrc/`` into ``librtprune.so`` and return its path."""
    cmd = [HIPCC] + FLAGS + list(extra_flags) + ["-o", LIB_PATH] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True, extra_flags=sys.argv[1:]))
