"""Compile the HIP sources in csrc/ into paper_2410_05076_amd/libtidal.so for gfx950."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libtidal.so")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
    "-Wall", "-Wno-unused-function",
]


def build(extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.run([hipcc, *HIPCC_FLAGS, *extra, *SOURCES, "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(sys.argv[1:]))
