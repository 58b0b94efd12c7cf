"""The register SpDM kernel issues its B loads from asm statements and waits for them itself.
This test compiles every instance to assembly and proves, on the generated code, that no
compiler-generated instruction touches a register whose load may still be in flight, and that
nothing spills."""
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2005_14469_amd import build
from paper_2005_14469_amd import isa_check

CSRC = build.CSRC
ROOT = build.ROOT


def _compile(v: int) -> str:
    src = os.path.join(CSRC, f"spdm_sched_v{v}.hip")
    out = os.path.join(tempfile.mkdtemp(prefix="gcoo_isa_"), f"v{v}.s")
    subprocess.check_call(["hipcc", *build.FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S",
                           "--cuda-device-only", "-o", out, src], stderr=subprocess.DEVNULL)
    return open(out).read()


@pytest.fixture(scope="module")
def asm():
    with ThreadPoolExecutor(max_workers=3) as ex:
        texts = list(ex.map(_compile, (4, 2, 1)))
    return dict(zip((4, 2, 1), texts))


@pytest.mark.parametrize("v", [4, 2, 1])
def test_no_compiler_instruction_touches_a_register_with_a_load_in_flight(asm, v):
    regs, bad = isa_check.check(asm[v], f"_ZN4gcoo10spdm_schedILi{v}E")
    assert len(regs) >= 4 * v          # the check found the asm loads
    assert not bad, bad[:10]


@pytest.mark.parametrize("v", [4, 2, 1])
def test_no_scratch_and_two_waves_per_simd(asm, v):
    text = asm[v]
    meta = text[text.index("amdhsa.kernels"):]
    get = lambda key: int(re.search(rf"\.{key}:\s+(\d+)", meta).group(1))
    assert get("vgpr_spill_count") == 0
    assert get("sgpr_spill_count") <= 16        # scalar spills go to lanes of a spare VGPR, not to memory
    assert get("private_segment_fixed_size") == 0
    assert get("vgpr_count") <= 256


def test_checker_sees_a_planted_violation(asm):
    """The checker itself: a compiler-style copy out of a load destination, planted right after the
    first asm load, must be reported."""
    text = asm[4]
    regs, bad = isa_check.check(text, "_ZN4gcoo10spdm_schedILi4E")
    assert not bad
    first = text.index("global_load_dwordx4")
    dst = int(re.match(r"global_load_dwordx4 v\[(\d+):", text[first:]).group(1))
    end_asm = text.index("#ASMEND", first)
    eol = text.index("\n", end_asm)
    planted = text[:eol + 1] + f"\tv_mov_b32_e32 v0, v{dst}\n" + text[eol + 1:]
    _, bad2 = isa_check.check(planted, "_ZN4gcoo10spdm_schedILi4E")
    assert bad2
    # a wait that lets one load too many stay in flight is seen as well
    waits = sorted({int(n) for n in re.findall(r"s_waitcnt vmcnt\((\d+)\)", text)})
    assert len(waits) >= 3
    n = waits[-1]
    loosened = text.replace(f"s_waitcnt vmcnt({n})", f"s_waitcnt vmcnt({n + 1})")
    _, bad3 = isa_check.check(loosened, "_ZN4gcoo10spdm_schedILi4E")
    assert bad3
