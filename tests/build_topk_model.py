"""Compile tests/topk_model.cpp (the CPU model of the top-k kernels' index arithmetic) with g++."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "topk_model.cpp")
LIB = os.path.join(HERE, "libtopk_model.so")
HEADER = os.path.join(ROOT, "paper_2410_05076_amd", "csrc", "topk_math.h")


def build(force=True):
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= max(os.path.getmtime(SRC), os.path.getmtime(HEADER))):
        return LIB
    subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
                    "-I", os.path.dirname(HEADER), SRC, "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
