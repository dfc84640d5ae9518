"""Builds libqgemm.so (HIP, gfx950 only) in-tree with one hipcc command."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqgemm.so")
SOURCES = ["api.hip", "pack.hip", "quantize_a.hip", "gemm_tile.hip", "gemm_skinny.hip", "conv_group.hip", "conv_patch.hip"]
PROBES_SRC = os.path.join(ROOT, "bench_probes.hip")   # bench.py's measurement probes, a library of their own
PROBES_LIB = os.path.join(ROOT, "libbench_probes.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # the fp32 requantization sequence must not be fused
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading scalar kernel arguments arrive in scalar registers with the wave (the microsecond kernels declare
    # what they need first that way); kernels whose first argument is a struct are unaffected
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def build_lib(verbose=False, extra=(), incremental=False):
    """One object per source file (compiled in parallel), then one link.  incremental=True recompiles only the
    sources that are newer than their object (or older than a header); the default compiles everything."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".inc"))]
    headers.append(os.path.join(ROOT, "include", "qgemm.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    procs, objs = [], []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        if incremental and not extra and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        cmd = ["hipcc"] + compile_flags + list(extra) + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd)))
    for cmd, pr in procs:
        if pr.wait() != 0:
            raise subprocess.CalledProcessError(pr.returncode, cmd)
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


def build_probes(verbose=False):
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", PROBES_SRC, "-o", PROBES_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return PROBES_LIB


if __name__ == "__main__":
    inc = "--incremental" in sys.argv[1:]
    build_lib(verbose=True, extra=[a for a in sys.argv[1:] if a != "--incremental"], incremental=inc)
    build_probes(verbose=True)
    print("built", LIB)
