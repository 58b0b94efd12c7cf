"""What each part of the workgroup-shared SpDM kernel costs: the kernel is rebuilt with one or more of its parts
taken out (GCOO_SHARE_ABLATE in csrc/gcoo_spdm_share_kernel.hpp) and every variant is timed on the same workload.

    python -m paper_2005_14469_amd.microbench.ablate --build      (no GPU needed: compiles the variants)
    python -m paper_2005_14469_amd.microbench.ablate --run [--workload config3]

An ablated kernel computes wrong products (that is the point: only its time is read); all its addresses are
formed exactly as in the whole kernel.  The variants are libraries of their own beside this file
(libgcoo_ablate_<bits>.so): nothing else loads them.  Each one is timed by bench.py in a process of its own,
which loads it in place of libgcoo.so through the GCOO_LIBRARY variable."""
import json
import os
import subprocess
import sys

from .. import build

HERE = os.path.dirname(os.path.abspath(__file__))

# (bits of GCOO_SHARE_ABLATE, what is taken out)
VARIANTS = [
    (0, "nothing: the whole kernel"),
    (1, "the requests for the rows of B"),
    (2, "the multiply-adds"),
    (16, "nothing, but the wait in front of the barrier leaves two bands' rows in flight"),
    (1 | 2, "requests and multiply-adds"),
    (1 | 4, "requests and the barrier between bands"),
    (1 | 2 | 4, "requests, multiply-adds and barrier"),
    (1 | 2 | 8, "requests, multiply-adds and the singles' reads of B values from LDS"),
    (1 | 2 | 4 | 8, "all of these: what is left is the walk over bands, headers and record blocks"),
]


def lib_path(bits: int) -> str:
    return os.path.join(HERE, f"libgcoo_ablate_{bits}.so")


def compile_variants() -> None:
    build.build()                                   # the other translation units, and the checked whole kernel
    src = os.path.join(build.CSRC, "spdm_share.hip")
    others = [os.path.join(build.OBJ, os.path.basename(s)[:-4] + ".o") for s in build.sources() if s != src]
    for bits, _ in VARIANTS:
        obj = os.path.join(build.OBJ, f"spdm_share_ablate_{bits}.o")
        subprocess.check_call(["hipcc", *build.FLAGS, f"-DGCOO_SHARE_ABLATE={bits}", "-I", os.path.join(build.ROOT, "include"),
                               "-I", build.CSRC, "-c", src, "-o", obj])
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path(bits), obj, *others])
        print(lib_path(bits), flush=True)


def time_variant(bits: int, workload: str) -> float:
    env = dict(os.environ, GCOO_LIBRARY=lib_path(bits))
    out = subprocess.run([sys.executable, os.path.join(build.ROOT, "bench.py"), "--workload", workload, "--share", "always",
                          "--variant", "3", "--p", "42", "--steps", "30", "--warmup", "3", "--no-cpu", "--no-dense",
                          "--secondary", ""], env=env, check=True, capture_output=True, text=True, timeout=300).stdout
    line = [ln for ln in out.splitlines() if ln.startswith("{")][-1]
    return float(json.loads(line)["spdm"]["ms"])


def run(workload: str) -> None:
    missing = [lib_path(b) for b, _ in VARIANTS if not os.path.exists(lib_path(b))]
    if missing:
        raise SystemExit(f"not built: {missing[0]} (run with --build first)")
    print(f"spdm_share on {workload}, p = 42: mean kernel time of 30 launches with parts of the kernel taken out", flush=True)
    for bits, what in VARIANTS:
        print(f"  ablate={bits:<2d} {time_variant(bits, workload):8.4f} ms   without {what}", flush=True)


if __name__ == "__main__":
    args = sys.argv[1:]
    if "--build" in args:
        compile_variants()
    if "--run" in args:
        run(args[args.index("--workload") + 1] if "--workload" in args else "config3")
    if "--build" not in args and "--run" not in args:
        raise SystemExit(__doc__)
