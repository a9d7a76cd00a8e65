"""Builds libdlc.so (HIP, gfx950 only) in-tree with hipcc: one object per source file, in parallel, then a link."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libdlc.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + [os.path.join(ROOT, "include", "dlc.h")]

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-ffp-contract=off",                                         # the quantiser is one rounded operation at a time
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed fp32 instructions
    "-Wall", "-Wno-unused-function",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def _compile(hipcc: str, src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
    cmd = [hipcc, *FLAGS, "-c", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"), "-o", obj, src]
    subprocess.run(cmd, check=True)
    return obj


def build(force: bool = True) -> str:
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        os.makedirs(OBJ_DIR, exist_ok=True)
        jobs = min(8, len(SOURCES), os.cpu_count() or 1)
        with ThreadPoolExecutor(max_workers=jobs) as ex:
            objs = list(ex.map(lambda s: _compile(hipcc, s), SOURCES))
        subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
