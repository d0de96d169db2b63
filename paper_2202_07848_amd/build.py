"""Builds libckpt.so (HIP, gfx950 only) next to this file.

    python -m paper_2202_07848_amd.build

hipcc cross-compiles without a GPU.  The library is built in-tree so that it
travels with the source tree; it is not installed anywhere.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libckpt.so")
SOURCES = ["api.hip", "fingerprint.hip", "diff_scan.hip", "copy.hip", "match.hip",
           "transport.hip", "swap.hip", "exchange.hip", "chain.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-fno-gpu-rdc", "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed-fp32 VALU forms stay off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = False, extra=()) -> str:
    cmd = [HIPCC] + FLAGS + list(extra) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the packed-fp32 target feature and says so once per
    # kernel; that note is expected and carries no information
    noise = "'-packed-fp32-ops' is not a recognized feature for this target"
    for line in proc.stdout.splitlines():
        if noise not in line:
            print(line, flush=True)
    if proc.returncode != 0:
        raise subprocess.CalledProcessError(proc.returncode, cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
