"""Compile the C oracle into oracle/libtidal_oracle.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "tidal_oracle.c")
LIB = os.path.join(HERE, "libtidal_oracle.so")

# x86-64-v3 (AVX2) rather than -march=native: the library is built in one
# container and run on another host.  -ffp-contract=off keeps every multiply
# and add a separate fp32 operation, in the order the source states.
CFLAGS = ["-O2", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
          "-std=c11", "-Wall", "-Wextra"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    subprocess.run(["gcc", *CFLAGS, SRC, "-o", LIB, "-lm"], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
