"""Build-time check of the device code the compiler made from csrc/galv_dp.hip.

The sweep kernel requests its next group of transition keys with hand-issued scalar loads
(`s_load_dwordx16 / x8 / x4` inside inline asm) and waits for them later, after the arithmetic on the
current group.  The compiler does not know that such a load is still in flight: to it the
destination registers are defined as soon as the asm statement ends.  Under scalar-register
pressure it could therefore spill those registers (saving stale contents) or reuse them for
something else, such as an address, before the data lands - wrong keys at best, a wild
pointer at worst.  Nothing in the language forbids that, so the build verifies it on the
produced ISA: between every scalar load that sits inside an inline-asm block and the next `s_waitcnt` with `lgkmcnt(0)`
no instruction may name one of the load's destination registers, and control may not leave
the straight line (no label, no branch).  A tile shape or flag that makes the compiler break
this fails the build instead of reaching a GPU.
"""
from __future__ import annotations

import re

_LOAD = re.compile(r"\s*s_load_dwordx(?:4|8|16)\s+s\[(\d+):(\d+)\]")
_RANGE = re.compile(r"\bs\[(\d+):(\d+)\]")
_SINGLE = re.compile(r"\bs(\d+)\b")
_FLOW = re.compile(r"\s*(s_cbranch|s_branch|s_endpgm|s_setpc|s_swappc|s_call)")


def _sgprs(text: str) -> set:
    regs = set()
    for m in _RANGE.finditer(text):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in _SINGLE.finditer(text):
        regs.add(int(m.group(1)))
    return regs


def scalar_prefetch_violations(asm_text: str) -> list:
    """Violations as (function, load line number, offending line number, text)."""
    lines = asm_text.split("\n")
    out, func, in_asm = [], "?", False
    for i, line in enumerate(lines):
        head = line.split(";")[0].rstrip()
        if head.endswith(":") and head[:1] not in (" ", "\t", "."):
            func = head[:-1]
        if "#ASMSTART" in line:
            in_asm = True
        elif "#ASMEND" in line:
            in_asm = False
        m = _LOAD.match(line)
        if not m or not in_asm:        # only loads written by hand (inside inline asm) are at risk:
            continue                   # the compiler waits for its own before it touches their registers
        dst = set(range(int(m.group(1)), int(m.group(2)) + 1))
        j = i + 1
        while j < len(lines):
            code = lines[j].split(";")[0].strip()
            j += 1
            if not code or code.startswith("."):
                if code.startswith(".LBB"):
                    out.append((func, i + 1, j, "label before the wait: " + code))
                    break
                continue
            if code.startswith("s_waitcnt") and "lgkmcnt(0)" in code:
                break
            if code.endswith(":") or _FLOW.match(code):
                out.append((func, i + 1, j, "control flow before the wait: " + code))
                break
            if _LOAD.match(code):
                continue                      # a sibling request of the same group
            if _sgprs(code) & dst:
                out.append((func, i + 1, j, code))
        else:
            out.append((func, i + 1, len(lines), "no wait found"))
    return out


def count_requests(asm_text: str) -> int:
    n, in_asm = 0, False
    for line in asm_text.split("\n"):
        if "#ASMSTART" in line:
            in_asm = True
        elif "#ASMEND" in line:
            in_asm = False
        elif in_asm and _LOAD.match(line):
            n += 1
    return n
