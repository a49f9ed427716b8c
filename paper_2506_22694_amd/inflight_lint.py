"""Build-time check of the gfx950 assembly of the draft-step kernels: nothing touches a register that a
hand-issued load still has in flight.

The draft-step kernels issue their global loads from inline assembly and wait for them with
`s_waitcnt vmcnt(N)` statements of their own, many instructions later.  Between the two the compiler
believes the destination registers already hold their values: a register copy it places there (at the
join of a branch, when it splits a live range, for a spill) would read data that has not arrived.  This
module reads the device assembly the compiler produced and follows every path from each such load to the
first wait that is certain to cover it; any instruction on the way that names one of the load's
destination registers is reported.

Model: loads return in the order they were issued, so after `s_waitcnt vmcnt(N)` a load is complete if at
least N vector-memory loads were issued after it (stores and atomics are not counted: they may complete
out of order with loads, which can only make the wait stronger than assumed here).
"""
from __future__ import annotations

import re
import sys
from dataclasses import dataclass, field

_VREG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
_VMCNT = re.compile(r"vmcnt\((\d+)\)")
_LABEL = re.compile(r"^([.\w$]+):")
_LOADS = ("global_load", "buffer_load", "flat_load", "scratch_load")
_CAP = 64           # vmcnt holds 6 bits: a wait with any N covers a load with this many loads behind it


@dataclass
class Ins:
    text: str
    line: int
    by_hand: bool
    regs: frozenset = field(default_factory=frozenset)


def _regs(text: str) -> frozenset:
    out = set()
    for m in _VREG.finditer(text):
        if m.group(1) is not None:
            out.add(int(m.group(1)))
        else:
            out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return frozenset(out)


def _functions(asm: str):
    """Yields (name, [Ins], {label: index}) for every function of an assembly file."""
    name, ins, labels, by_hand = None, [], {}, False
    for no, raw in enumerate(asm.splitlines(), 1):
        s = raw.strip()
        if s.startswith(";;#ASMSTART"):
            by_hand = True
            continue
        if s.startswith(";;#ASMEND"):
            by_hand = False
            continue
        s = s.split(";")[0].strip()
        if not s:
            continue
        m = _LABEL.match(s)
        if m:
            lab = m.group(1)
            if not lab.startswith(".L") and name is None:
                name, ins, labels = lab, [], {}
            elif name is not None:
                labels[lab] = len(ins)
            continue
        if s.startswith("."):
            if s.startswith(".Lfunc_end") or s.startswith(".size"):
                pass
            continue
        if name is None:
            continue
        ins.append(Ins(s, no, by_hand, _regs(s.split(None, 1)[1]) if " " in s or "\t" in s else frozenset()))
        if s.startswith("s_endpgm"):
            yield name, ins, labels
            name = None
    if name is not None and ins:
        yield name, ins, labels


def _successors(ins, labels, i):
    t = ins[i].text
    op = t.split()[0]
    if op.startswith("s_endpgm") or op.startswith("s_setpc"):
        return []
    if op == "s_branch":
        return [labels[t.split()[1]]]
    if op.startswith("s_cbranch"):
        return [labels[t.split()[-1]], i + 1]
    return [i + 1]


def check_function(name, ins, labels, drains=None):
    """Violations of one function: (function, line of the load, line of the instruction, its text).

    drains (a set, optional) collects (function, line, text) of waits the COMPILER inserted that are the first
    to cover a hand-issued load: legal, but such a wait also holds up every older hand-issued load, so inside a
    prefetch pipeline it is worth a look (a performance remark, not an error)."""
    bad = []
    for i, x in enumerate(ins):
        if not (x.by_hand and x.text.startswith(_LOADS)):
            continue
        dest = _regs(x.text.split(",")[0])
        seen = set()
        todo = [(j, 0) for j in _successors(ins, labels, i)]
        while todo:
            j, behind = todo.pop()
            if j >= len(ins) or (j, behind) in seen:
                continue
            seen.add((j, behind))
            y = ins[j]
            op = y.text.split()[0]
            if op == "s_waitcnt":
                m = _VMCNT.search(y.text)
                if m and behind >= int(m.group(1)):
                    if drains is not None and not y.by_hand:
                        drains.add((name, y.line, y.text))
                    continue                      # the load has landed on this path
            elif y.regs & dest:
                bad.append((name, x.line, y.line, y.text))
                continue
            if op.startswith(_LOADS):
                behind = min(behind + 1, _CAP)
            todo.extend((s, behind) for s in _successors(ins, labels, j))
    return bad


def check_asm(asm: str, drains=None):
    """All violations in an assembly file, and the number of hand-issued loads that were followed."""
    bad, loads = [], 0
    for name, ins, labels in _functions(asm):
        loads += sum(1 for x in ins if x.by_hand and x.text.startswith(_LOADS))
        bad.extend(check_function(name, ins, labels, drains))
    return bad, loads


if __name__ == "__main__":
    status = 0
    for path in sys.argv[1:]:
        compiler_waits = set()
        violations, n = check_asm(open(path).read(), compiler_waits)
        print(f"{path}: {n} hand-issued loads, {len(violations)} violations, "
              f"{len(compiler_waits)} compiler-inserted waits that cover hand-issued loads")
        for v in violations[:20]:
            print("  ", v)
        for v in sorted(compiler_waits)[:20]:
            print("   remark:", v)
        status |= bool(violations)
    sys.exit(status)
