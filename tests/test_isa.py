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


INSTANCES = ("4", "4t", "2")        # columns per lane; t = the tall accumulator file


def _kernels(v: str):
    return build.sched_kernel_names(f"spdm_sched_v{v}")


def _compile(v: str) -> str:
    src = os.path.join(CSRC, f"spdm_sched_v{v}.hip")
    out = os.path.join(tempfile.mkdtemp(prefix="gcoo_isa_"), f"v{v}.s")
    subprocess.check_call(["hipcc", *build.FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S",
                           "--cuda-device-only", "-o", out, src], stderr=subprocess.DEVNULL)
    return open(out).read()


@pytest.fixture(scope="module")
def asm():
    with ThreadPoolExecutor(max_workers=4) as ex:
        texts = list(ex.map(_compile, INSTANCES))
    return dict(zip(INSTANCES, texts))


@pytest.mark.parametrize("v", INSTANCES)
def test_no_compiler_instruction_touches_a_register_with_a_load_in_flight(asm, v):
    for kernel in _kernels(v):
        regs, bad = isa_check.check(asm[v], kernel)
        assert len(regs) >= 4 * int(v.rstrip("t"))          # the check found the asm loads
        assert not bad, bad[:10]


@pytest.mark.parametrize("v", INSTANCES)
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
    text = asm["4"]
    K = _kernels("4")[0]
    regs, bad = isa_check.check(text, K)
    assert not bad
    start = re.search(rf"^{re.escape(K)}\w*:", text, re.M).start()          # inside the kernel that is checked
    first = text.index("global_load_dwordx4", start)
    dst = int(re.match(r"global_load_dwordx4 v\[(\d+):", text[first:]).group(1))
    end_asm = text.index("#ASMEND", first)
    eol = text.index("\n", end_asm)
    planted = text[:eol + 1] + f"\tv_mov_b32_e32 v0, v{dst}\n" + text[eol + 1:]
    _, bad2 = isa_check.check(planted, K)
    assert bad2
    # a wait that lets one load too many stay in flight is seen as well
    waits = sorted({int(n) for n in re.findall(r"s_waitcnt vmcnt\((\d+)\)", text)})
    assert len(waits) >= 3
    n = waits[-1]
    loosened = text.replace(f"s_waitcnt vmcnt({n})", f"s_waitcnt vmcnt({n + 1})")
    _, bad3 = isa_check.check(loosened, K)
    assert bad3


# ------------------------------------------------------------------ the workgroup-shared kernel's loads straight to LDS

SHARE = "_ZN4gcoo10spdm_share"


@pytest.fixture(scope="module")
def share_asm():
    src = os.path.join(CSRC, "spdm_share.hip")
    out = os.path.join(tempfile.mkdtemp(prefix="gcoo_isa_"), "share.s")
    subprocess.check_call(["hipcc", *build.FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S",
                           "--cuda-device-only", "-o", out, src], stderr=subprocess.DEVNULL)
    return open(out).read()


def test_share_kernel_does_not_spill_and_keeps_its_occupancy(share_asm):
    assert [int(x) for x in re.findall(r"\.vgpr_spill_count:\s+(\d+)", share_asm)] == [0]
    assert [int(x) for x in re.findall(r"\.vgpr_count:\s+(\d+)", share_asm)] == [256]          # two waves per SIMD
    assert [int(x) for x in re.findall(r"\.private_segment_fixed_size:\s+(\d+)", share_asm)] == [0]


def test_every_load_to_lds_sets_m0_itself_and_at_most_six_cross_a_barrier(share_asm):
    loads, problems = isa_check.check_lds_loads(share_asm, SHARE, in_flight=6)
    assert loads >= 2 + 3 * 6 + 5        # two ring pieces and three bands of six rows in the text, a ring piece per block advance
    assert not problems, problems
    # the same text judged by the strict rule (nothing in flight at a barrier) is refused: the kernel does
    # keep the rows of the band after next on their way
    _, strict = isa_check.check_lds_loads(share_asm, SHARE)
    assert strict and "barrier" in strict[0]


def test_lds_load_checker_sees_planted_mistakes(share_asm):
    i = share_asm.index(SHARE)
    head, body = share_asm[:i], share_asm[i:]
    # an M0 write taken away: the load behind it would use what the one before left (or the index mode's row)
    # (one right behind the index mode: the walk back from its loads then ends there)
    m = re.search(r"(s_set_gpr_idx_off\n\s*)(s_mov_b32 m0, s72)", body)
    _, problems = isa_check.check_lds_loads(head + body.replace(m.group(0), m.group(1) + "s_nop 0", 1), SHARE, in_flight=6)
    assert problems and "M0" in problems[0]
    # an index-mode instruction between the M0 write and the load
    m = re.search(r"(s_mov_b32 m0, s\d+\n)", body)
    _, problems = isa_check.check_lds_loads(head + body.replace(m.group(1), m.group(1) + "\ts_set_gpr_idx_off\n", 1), SHARE, in_flight=6)
    assert problems and "M0" in problems[0]
    # the wait before a barrier weakened to one that leaves more row loads in flight than the kernel may
    weakened = body.replace("s_waitcnt vmcnt(6)\n\ts_barrier", "s_waitcnt vmcnt(7)\n\ts_barrier")
    assert weakened != body
    _, problems = isa_check.check_lds_loads(head + weakened, SHARE, in_flight=6)
    assert problems and "barrier" in problems[0]
