"""Builds libpconv.so (host packer + gfx950 kernels) in-tree with hipcc.  Cross-compiles without a GPU."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpconv.so")
PEAKS_LIB = os.path.join(HERE, "libpconv_peaks.so")
SOURCES = ["pconv_host.cpp", "pconv_device.hip", "pconv_mfma.hip", "pconv_admm.hip", "pconv_backward.hip"]

# Packed fp32 instructions are switched off for every HIP translation unit of this project.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-pass-failed",
]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    # per-pattern code sections of the tiled kernel (generated source, not committed)
    sys.path.insert(0, CSRC)
    try:
        import gen_pattern_leaves
        gen_pattern_leaves.main(os.path.join(CSRC, "pattern_leaves.inc"))
    finally:
        sys.path.pop(0)
    # one object per source, compiled side by side (the matrix-core kernel's instantiations alone take minutes), then
    # one link; the objects live in a build folder that is not committed
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if verbose and out.strip():
            print(out)

    def compile_one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        run([hipcc, *flags, "-c", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-o", obj, os.path.join(CSRC, src)])
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), max(1, (os.cpu_count() or 2) - 1))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    run([hipcc, "-shared", "--offload-arch=gfx950", "-o", LIB, *objs])
    # the measured-peaks kernels: a library of their own, not linked into libpconv.so
    cmd = [hipcc, *HIPCC_FLAGS, "-I" + os.path.join(ROOT, "include"), "-o", PEAKS_LIB, os.path.join(CSRC, "pconv_peaks.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
