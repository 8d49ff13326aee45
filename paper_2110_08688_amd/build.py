"""Build libmggcn.so (HIP, gfx950 only) in-tree with hipcc.  Cross-compiles without a GPU."""
from __future__ import annotations

import concurrent.futures as cf
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmggcn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 VALU forms are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    deps = [src] + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "mggcn.h")]
    if os.path.exists(obj) and all(os.path.getmtime(obj) > os.path.getmtime(d) for d in deps):
        if not os.environ.get("MGGCN_FORCE_REBUILD"):
            return obj
    subprocess.check_call([HIPCC, *FLAGS, "-c", src, "-o", obj])
    return obj


def build(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    if force:
        os.environ["MGGCN_FORCE_REBUILD"] = "1"
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    try:
        with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
            objs = list(ex.map(_compile, srcs))
    finally:
        os.environ.pop("MGGCN_FORCE_REBUILD", None)
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs])
    build_probes()
    return LIB


def build_probes() -> list:
    """Stand-alone measurement programs (probes/*.hip -> probes/<name>): not linked into the library."""
    outs = []
    for src in sorted(glob.glob(os.path.join(HERE, "probes", "*.hip"))):
        exe = src[: -len(".hip")]
        subprocess.check_call([HIPCC, *[f for f in FLAGS if f != "-fPIC"], "-o", exe, src])
        outs.append(exe)
    return outs


if __name__ == "__main__":
    import sys

    print(build(force="--force" in sys.argv))
