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


def _checked(src: str) -> bool:
    """Sources whose generated code is verified by isa_check (kernels that issue loads from asm)."""
    return os.path.basename(src).startswith("spdm_sched_v")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
    extra = ["-save-temps=obj"] if _checked(src) else []      # keeps the device assembly next to the object
    subprocess.check_call(["hipcc", *FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj])
    return obj


def verify_generated_code() -> None:
    """Refuse to link a library whose asm-issued loads are not provably safe.

    The register SpDM kernel keeps loads in flight behind the compiler's back; isa_check proves
    on the assembly that no instruction touches a register before a wait has covered its load.
    A compiler change (or a careless edit) that breaks this would read stale registers or, worse,
    use them as addresses, so the check is part of the build, not only of the tests.
    """
    from . import isa_check
    for src in sources():
        if not _checked(src):
            continue
        stem = os.path.basename(src)[:-4]
        asm = os.path.join(OBJ, f"{stem}-hip-amdgcn-amd-amdhsa-gfx950.s")
        text = open(asm).read()
        v = stem.rsplit("v", 1)[1]
        for kernel in (f"_ZN4gcoo10spdm_schedILi{v}E", f"_ZN4gcoo15spdm_sched_coopILi{v}E"):
            regs, bad = isa_check.check(text, kernel)
            if not regs:
                raise RuntimeError(f"{stem}: no asm-issued loads found in {kernel} (check is blind)")
            if bad:
                raise RuntimeError(f"{stem} {kernel}: {len(bad)} instructions touch registers with a load in flight, e.g. {bad[:3]}")


def build(force: bool = True, jobs: int = 8) -> str:
    if force or stale():
        os.makedirs(OBJ, exist_ok=True)
        with ThreadPoolExecutor(max_workers=jobs) as ex:
            objs = list(ex.map(_compile, sources()))
        verify_generated_code()
        tmp = LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
