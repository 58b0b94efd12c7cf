"""Compile the HIP library (csrc/*.hip -> libgcoo.so) for gfx950 with hipcc.  No GPU is needed.

Every .hip file is one translation unit; they are compiled in parallel and linked into one
shared library.
"""
from __future__ import annotations

import glob
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgcoo.so")
# the CSR row-split routine the benchmark compares against: a library of its own, not part of the GCOO path
BASELINE_SRC = os.path.join(HERE, "csrc_baseline", "csr_baseline.hip")
BASELINE_LIB = os.path.join(HERE, "libgcoo_baseline.so")

# Packed fp32 VALU instructions are switched off for every kernel of this library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-Wno-inline-asm"]      # the index-mode asm statements name M0 as clobbered, which clang remarks on


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _deps():
    return sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + [os.path.join(ROOT, "include", "gcoo.h"), BASELINE_SRC,
                                                                  os.path.join(ROOT, "include", "gcoo_baseline.h")]


def stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(BASELINE_LIB):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(BASELINE_LIB))
    return any(os.path.getmtime(f) > t for f in _deps())


def _checked(src: str) -> bool:
    """Sources whose generated code is verified by isa_check (kernels that issue loads from asm, or that
    load straight to LDS next to the index mode)."""
    name = os.path.basename(src)
    return name.startswith("spdm_sched_v") or name == "spdm_share.hip"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
    extra = ["-save-temps=obj"] if _checked(src) else []      # keeps the device assembly next to the object
    subprocess.check_call(["hipcc", *FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj])
    return obj


def sched_kernel_names(stem: str):
    """Mangled name prefixes of the kernels in spdm_sched_v<V>[t].hip (t = the tall accumulator layout)."""
    v = stem.rsplit("v", 1)[1]
    if v.endswith("t"):                  # that layout has no workgroup-shared kernel
        return (f"_ZN4gcoo8acc_tall10spdm_schedILi{v[:-1]}E",)
    return (f"_ZN4gcoo7acc_std10spdm_schedILi{v}E", f"_ZN4gcoo7acc_std15spdm_sched_coopILi{v}E")


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
        if stem == "spdm_share":
            verify_share_code(stem, text)
            continue
        for kernel in sched_kernel_names(stem):
            regs, bad = isa_check.check(text, kernel)
            if not regs:
                raise RuntimeError(f"{stem}: no asm-issued loads found in {kernel} (check is blind)")
            if bad:
                raise RuntimeError(f"{stem} {kernel}: {len(bad)} instructions touch registers with a load in flight, e.g. {bad[:3]}")


def verify_share_code(stem: str, text: str) -> None:
    """The workgroup-shared kernel: no register spills, all 256 VGPRs (two waves per SIMD), every load that
    writes LDS sets M0 itself, and in front of every barrier a wait that leaves at most the six row loads of
    the band after next in flight."""
    from . import isa_check
    kernel = "_ZN4gcoo10spdm_share"
    if not isa_check.kernel_body(text, kernel):
        raise RuntimeError(f"{stem}: kernel {kernel} not found")
    loads, problems = isa_check.check_lds_loads(text, kernel, in_flight=6)
    if not loads:
        raise RuntimeError(f"{stem} {kernel}: no loads to LDS found (check is blind)")
    if problems:
        raise RuntimeError(f"{stem} {kernel}: {problems[:3]}")
    spills = [int(x) for x in re.findall(r"\.vgpr_spill_count:\s+(\d+)", text)]
    if len(spills) != 1 or any(spills):
        raise RuntimeError(f"{stem}: register spills {spills}")


def build(force: bool = True, jobs: int = 8) -> str:
    if force or stale():
        os.makedirs(OBJ, exist_ok=True)
        with ThreadPoolExecutor(max_workers=jobs) as ex:
            objs = list(ex.map(_compile, sources()))
        verify_generated_code()
        tmp = LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
        tmp = BASELINE_LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["hipcc", *FLAGS, "-shared", "-I", os.path.join(ROOT, "include"), BASELINE_SRC, "-o", tmp])
        os.replace(tmp, BASELINE_LIB)
    return LIB


def build_host_sanitized(jobs: int = 8) -> str:
    """A checking build: the same sources with the address and undefined-behaviour sanitizers on the HOST
    code only (the device code is compiled as usual), as _build/san/libgcoo.so.  For one pass of the tests that
    need no GPU; the command is printed by `python -m paper_2005_14469_amd.build --host-sanitize`."""
    out_dir = os.path.join(OBJ, "san")
    os.makedirs(out_dir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f if f != "-O3" else "-O1" for f in FLAGS] + ["-g"]

    def one(src):
        obj = os.path.join(out_dir, os.path.basename(src)[:-4] + ".o")
        subprocess.check_call(["hipcc", *flags, *san, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj])
        return obj
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(one, sources()))
    lib = os.path.join(out_dir, "libgcoo.so")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *san[:4], "-shared-libsan", "-o", lib, *objs])
    return lib


if __name__ == "__main__":
    import sys
    if "--host-sanitize" in sys.argv[1:]:
        lib = build_host_sanitized()
        rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        print(lib)
        print(f"run: GCOO_LIBRARY={lib} LD_PRELOAD={rt[0] if rt else '<libclang_rt.asan-x86_64.so>'} ASAN_OPTIONS=detect_leaks=0 "
              "UBSAN_OPTIONS=halt_on_error=1 python -m pytest tests/test_abi_host.py -q")
    else:
        print(build())
