"""Compiles csrc/ into libdistdl.so (gfx950) next to this file."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["plan.cpp", "profile.cpp", "halo.hip", "collective.hip", "conv.hip", "conv_mfma.hip", "conv_small.hip", "affine.hip", "gemm_mfma.hip", "glue.hip", "repart.hip", "convcp.hip"]
LIB = os.path.join(HERE, "libdistdl.so")


def build(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-shared", "-fPIC", "-O3", "-std=c++17", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-result", "-Wno-unknown-warning-option",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    for s in SOURCES:
        if s.endswith(".cpp"):
            cmd += ["-x", "hip", os.path.join(HERE, "csrc", s)]
        else:
            cmd.append(os.path.join(HERE, "csrc", s))
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
