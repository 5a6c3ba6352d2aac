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


if __name__ == "__main__":
    import sys
    args = sys.argv[1:]
    inc = "--incremental" in args
    print(build([a for a in args if a != "--incremental"], incremental=inc))
