"""Build libcnn.so (the C-ABI GPU library) in-tree with hipcc for gfx950.

    python -m paper_1602_06709_amd.build [--force]

Every .hip file under csrc/ is compiled to an object and linked into
paper_1602_06709_amd/libcnn.so.  hipcc cross-compiles without a GPU.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcnn.so")
HEADER = os.path.join(os.path.dirname(HERE), "include", "cnn.h")

FLAGS = [
    "-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
    # packed-fp32 VALU forms are switched off for this target (host pass warns that it ignores the feature)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _deps_mtime():
    deps = [HEADER] + [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    return max(os.path.getmtime(d) for d in deps)


def is_current():
    return os.path.exists(LIB) and os.path.getmtime(LIB) >= _deps_mtime()


def _compile(src, force, extra, objdir=None):
    obj = os.path.join(objdir or OBJ, os.path.basename(src)[:-4] + ".o")
    hdr_m = max(os.path.getmtime(HEADER), os.path.getmtime(os.path.join(CSRC, "common.h")))
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src), hdr_m):
        return obj
    subprocess.run(["hipcc", *FLAGS, *extra, "-c", src, "-o", obj], check=True)
    return obj


def build(force=False, extra=(), jobs=4, out=None, objdir=None):
    """out / objdir: build a variant (extra -D flags) somewhere else without touching the in-tree library."""
    os.makedirs(objdir or OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, list(extra), objdir), sources()))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out or LIB, *objs], check=True)
    return out or LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
