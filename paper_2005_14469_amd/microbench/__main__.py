"""Build and run the ceilings micro-benchmark (ceilings.hip) on the GPU of this machine:
    python -m paper_2005_14469_amd.microbench
The executable is paper_2005_14469_amd/microbench/ceilings (built with --build-only where there is no GPU); its output is plain text, one line per measurement."""
import os
import subprocess
import sys

from .. import build

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(HERE, "ceilings")


def compile_() -> str:
    subprocess.check_call(["hipcc", *build.FLAGS, "-I", os.path.join(build.ROOT, "include"), "-I", build.CSRC,
                           os.path.join(HERE, "ceilings.hip"), "-o", EXE])
    return EXE


if __name__ == "__main__":
    exe = compile_()
    if "--build-only" in sys.argv[1:]:
        print(exe)
    else:
        sys.exit(subprocess.call([exe]))
