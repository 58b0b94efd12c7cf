"""Static check of the generated GCN code of a kernel that issues loads from asm statements.

The SpDM kernel starts its B loads (and the loads of its schedule stream) with `global_load_*`
inside asm statements and waits for them with its own `s_waitcnt vmcnt(n)`; the compiler does not
know that those destination registers are still in flight.  That is only correct if no
instruction - the compiler's or the kernel's own asm - touches such a register before a wait has
covered its load.  This module proves it on the assembly text:

  * the kernel is cut into basic blocks and a control-flow graph is built from the branch
    instructions (compiler branches and the labels inside asm statements alike);
  * vector-memory operations complete in order, so the abstract state at a point is the queue of
    operations that may still be outstanding, oldest first, each with the registers it will
    write (stores carry none).  A load or store appends an entry, `s_waitcnt vmcnt(n)` keeps the
    youngest n entries, and where paths join the queues are aligned at their young end and
    merged entry by entry (what is outstanding at distance i from the youngest on any path);
  * a forward data-flow pass runs this to a fixed point, then every instruction that names a
    register of an entry still in the queue - other than a new load into it - is reported.
"""
from __future__ import annotations

import re

_LABEL = re.compile(r"^(\.LBB\d+_\d+|\d+):")
_BRANCH = re.compile(r"^\s*(s_cbranch_\w+|s_branch)\s+(\S+)")


def _regs(text: str) -> set[int]:
    out: set[int] = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def kernel_body(asm_text: str, mangled_prefix: str) -> list[str]:
    lines = asm_text.split("\n")
    start = next(i for i, l in enumerate(lines) if l.startswith(mangled_prefix) and ":" in l)
    body = []
    for l in lines[start + 1:]:
        if l.startswith(".Lfunc_end"):
            break
        body.append(l)
    return body


def check(asm_text: str, mangled_prefix: str):
    """Returns (load destination registers, [(line number, instruction)] of offending instructions)."""
    body = kernel_body(asm_text, mangled_prefix)
    # instruction stream with asm flag; blocks start at labels and after branches
    insts = []          # (text, in_asm)
    in_asm = False
    for l in body:
        if "#ASMSTART" in l:
            in_asm = True
            continue
        if "#ASMEND" in l:
            in_asm = False
            continue
        t = l.split(";")[0].strip() if not l.strip().startswith(";") else ""
        if not t or t.startswith("."):
            m = _LABEL.match(l.strip())
            if not m:
                continue
            t = l.strip().split(";")[0].strip()
        insts.append((t, in_asm))
    load_regs: set[int] = set()
    for t, a in insts:
        if a and t.startswith("global_load"):
            load_regs |= _regs(t.split()[1].rstrip(","))
    # basic blocks
    blocks = []         # dict(label, insts=[(idx, text, in_asm)], succ=[...])
    cur = dict(labels=[], insts=[])
    for i, (t, a) in enumerate(insts):
        m = _LABEL.match(t)
        if m:
            if cur["insts"] or cur["labels"]:
                blocks.append(cur)
                cur = dict(labels=[], insts=[])
            cur["labels"].append(m.group(1))
            continue
        cur["insts"].append((i, t, a))
        if _BRANCH.match(t) or t.startswith("s_endpgm"):
            blocks.append(cur)
            cur = dict(labels=[], insts=[])
    if cur["insts"] or cur["labels"]:
        blocks.append(cur)
    # a block that is only labels merges into the next one
    merged = []
    pend = []
    for b in blocks:
        if not b["insts"]:
            pend += b["labels"]
            continue
        b["labels"] = pend + b["labels"]
        pend = []
        merged.append(b)
    blocks = merged

    # Numeric local labels (asm) may repeat: "1f"/"1b" resolve to the nearest one forward/backward.
    def resolve(bi: int, target: str):
        if target.startswith(".LBB"):
            for j, b in enumerate(blocks):
                if target in b["labels"]:
                    return j
            raise ValueError(f"label {target} not found")
        m = re.match(r"(\d+)([fb])$", target)
        if not m:
            raise ValueError(f"branch target {target}")
        rng = range(bi + 1, len(blocks)) if m.group(2) == "f" else range(bi, -1, -1)
        for j in rng:
            if m.group(1) in blocks[j]["labels"]:
                return j
        raise ValueError(f"local label {target} not found")

    for bi, b in enumerate(blocks):
        succ = []
        last = b["insts"][-1][1]
        m = _BRANCH.match(last)
        if m:
            succ.append(resolve(bi, m.group(2)))
            if m.group(1) != "s_branch" and bi + 1 < len(blocks):
                succ.append(bi + 1)
        elif not last.startswith("s_endpgm") and bi + 1 < len(blocks):
            succ.append(bi + 1)
        b["succ"] = succ

    CAP = 64
    VMEM = ("global_load", "global_store", "global_atomic", "buffer_load", "buffer_store", "flat_load", "flat_store",
            "scratch_load", "scratch_store")

    def transfer(b, queue, report=None):
        queue = list(queue)
        for i, t, a in b["insts"]:
            op = t.split()[0]
            if op == "s_waitcnt":
                m = re.search(r"vmcnt\((\d+)\)", t)
                if m:
                    n = int(m.group(1))
                    queue = queue[len(queue) - n:] if n < len(queue) else queue
                    if n == 0:
                        queue = []
                continue
            used = _regs(t)
            if op.startswith(VMEM):
                is_load = "_load" in op
                dst = _regs(t.split()[1].rstrip(",")) if is_load else set()
                if report is not None:
                    pending = set().union(*queue) if queue else set()
                    if (used - dst) & pending:                    # address/data operands must have arrived
                        report.append((i, t))
                queue.append(frozenset(dst))
                if len(queue) > CAP:
                    queue = [frozenset(queue[0] | queue[1])] + queue[2:]
                continue
            if report is not None and queue:
                pending = set().union(*queue)
                if used & pending:
                    report.append((i, t))
        return tuple(queue)

    def merge(q1, q2):
        if q1 is None:
            return q2
        n = max(len(q1), len(q2))
        p1 = (frozenset(),) * (n - len(q1)) + tuple(q1)
        p2 = (frozenset(),) * (n - len(q2)) + tuple(q2)
        return tuple(a | b for a, b in zip(p1, p2))

    entry = [None] * len(blocks)
    entry[0] = ()
    work = [0]
    while work:
        bi = work.pop()
        out = transfer(blocks[bi], entry[bi])
        for sj in blocks[bi]["succ"]:
            new = merge(entry[sj], out)
            if new != entry[sj]:
                entry[sj] = new
                work.append(sj)
    bad = []
    for bi, b in enumerate(blocks):
        if entry[bi] is not None:
            transfer(b, entry[bi], bad)
    return sorted(load_regs), bad


def check_lds_loads(asm_text: str, mangled_prefix: str, in_flight: int = 0):
    """Loads that write LDS directly (`global_load_lds_*`) in a kernel that also uses the VGPR index mode.

    Such a load takes the LDS address of lane 0 from M0, and `s_set_gpr_idx_on/idx` overwrite M0.
    Returns (number of such loads, list of problems).  Proved on the text, block by block:
      * walking back from every such load, an instruction that writes M0 as a plain destination
        (`s_mov_b32 m0`, `s_add_i32 m0`, ...) comes before any label, branch or index-mode instruction
        (other loads to LDS in between are passed over: they leave M0 as it is);
      * walking back from every `s_barrier`, an `s_waitcnt` that names vmcnt(n), n <= in_flight, comes before
        any such load (what a wave has sent to LDS has arrived before the other waves are let past the
        barrier, except the youngest in_flight loads, which a kernel may keep on their way on purpose).
    """
    body = [l.split(";")[0].strip() for l in kernel_body(asm_text, mangled_prefix)]
    body = [l for l in body if l]
    problems = []
    loads = 0
    for i, line in enumerate(body):
        if line.startswith("global_load_lds"):
            loads += 1
            j = i - 1
            while j >= 0:
                t = body[j]
                if re.match(r"^s_\w+\s+m0\b", t):
                    break
                if _LABEL.match(t) or _BRANCH.match(t) or t.startswith("s_set_gpr_idx"):
                    problems.append(f"line {i}: '{line}' has no M0 write of its own (stopped at '{t}')")
                    break
                j -= 1
            else:
                problems.append(f"line {i}: '{line}' has no M0 write before it")
        elif line.startswith("s_barrier"):
            j = i - 1
            while j >= 0:
                t = body[j]
                waited = re.search(r"vmcnt\((\d+)\)", t) if t.startswith("s_waitcnt") else None
                if waited and int(waited.group(1)) <= in_flight:
                    break
                if t.startswith("global_load_lds"):
                    problems.append(f"line {i}: barrier with a load to LDS ('{t}') not awaited")
                    break
                if _LABEL.match(t):            # the walk stays in the block: a barrier that opens a block is judged unsafe
                    if any(b.startswith("global_load_lds") for b in body):
                        problems.append(f"line {i}: barrier at the start of a block, no wait seen")
                    break
                j -= 1
    return loads, problems
