"""Compile the HIP library (csrc/*.hip -> libgcoo.so) for gfx950 with hipcc.  No GPU is needed.

Every .hip file is one translation unit; they are compiled in parallel and linked into one
shared library.
"""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgcoo.so")

# Packed fp32 VALU instructions are switched off for every kernel of this library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _deps():
    return sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + [os.path.join(ROOT, "include", "gcoo.h")]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in _deps())


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
    subprocess.check_call(["hipcc", *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj])
    return obj


def build(force: bool = True, jobs: int = 8) -> str:
    if force or stale():
        os.makedirs(OBJ, exist_ok=True)
        with ThreadPoolExecutor(max_workers=jobs) as ex:
            objs = list(ex.map(_compile, sources()))
        tmp = LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
