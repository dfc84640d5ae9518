"""Builds libqgemm.so (HIP, gfx950 only) in-tree with one hipcc command."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqgemm.so")
SOURCES = ["api.hip", "pack.hip", "quantize_a.hip", "gemm_tile.hip", "gemm_skinny.hip", "conv_group.hip", "probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # the fp32 requantization sequence must not be fused
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def build_lib(verbose=False, extra=()):
    cmd = ["hipcc"] + FLAGS + list(extra) + sources() + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_lib(verbose=True, extra=sys.argv[1:])
    print("built", LIB)
