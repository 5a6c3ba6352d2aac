"""Compile the HIP sources in csrc/ into paper_2410_05076_amd/libtidal.so for gfx950.

Every source is compiled to an object file of its own (in parallel), then linked; there are no device
calls across translation units, so no relocatable device code is needed."""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libtidal.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h")))

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
    "-Wall", "-Wno-unused-function",
]


def build(extra=(), incremental=False, jobs=None):
    """Compiles and links the library.  incremental: keep objects that are newer than their source and
    every header (for edit-compile loops; the default compiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in HEADERS)
    todo, objs = [], []
    for src in SOURCES:
        obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        fresh = (incremental and not extra and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh:
            todo.append((src, obj))

    def compile_one(job):
        src, obj = job
        subprocess.run([hipcc, *HIPCC_FLAGS, *extra, "-c", src, "-o", obj], check=True)

    workers = jobs or min(8, os.cpu_count() or 1, max(1, len(todo)))
    with ThreadPoolExecutor(workers) as pool:
        list(pool.map(compile_one, todo))
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], check=True)
    return LIB


def build_sanitized_host_check():
    """Builds tests/abi_host_check.cpp against the library with the host side of api.hip (argument checks,
    workspace layout, launch planning) compiled with AddressSanitizer and UndefinedBehaviorSanitizer; the
    device code and the other objects are the normal ones (build() must have run).  Returns the executable."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    api_obj = os.path.join(OBJ_DIR, "api_san.o")
    chk_obj = os.path.join(OBJ_DIR, "abi_host_check.o")
    exe = os.path.join(OBJ_DIR, "abi_host_check")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g"]
    subprocess.run([hipcc, *flags, *san, "-c", os.path.join(HERE, "csrc", "api.hip"), "-o", api_obj], check=True)
    subprocess.run([hipcc, "-O1", "-g", "-std=c++17", "-I", os.path.join(ROOT, "include"), *san, "-c", "-x", "c++",
                    os.path.join(ROOT, "tests", "abi_host_check.cpp"), "-o", chk_obj], check=True)
    others = [os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o") for src in SOURCES if not src.endswith("api.hip")]
    subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", chk_obj, api_obj,
                    *others, "-o", exe], check=True)
    return exe


if __name__ == "__main__":
    import sys
    args = sys.argv[1:]
    inc = "--incremental" in args
    print(build([a for a in args if a != "--incremental"], incremental=inc))
