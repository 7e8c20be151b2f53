"""Build-time check of the LDS rank kernel's pinned scalar registers.

forest_kernels_ranklds.hip keeps the split program in two sets of 16 scalar registers,
s[36:51] and s[52:67], and its evaluation statements leave a scalar load into one of them in
flight when they end.  That is only sound if no instruction the compiler generates between two
such statements reads or writes those registers.  The compiler is told so through the
statements' operands; this script checks that it obeyed, on the assembly of the very sources
that go into the library: inside every loop that holds an evaluation statement, outside the
statements themselves, s36..s67 must not appear.

The statements' writes of M0 (the LDS row offset of every entry) need no check: the compiler
reserves M0, keeps nothing in it across an inline-assembly statement and refuses it as a clobber.  When the check fails the build does not stop: it compiles the
kernel's conservative form, whose statements leave nothing in flight (see build.py).
"""
from __future__ import annotations

import os
import re
import subprocess
import sys

_PINNED = re.compile(r"\bs(3[6-9]|4[0-9]|5[0-9]|6[0-7])\b|s\[(3[6-9]|4\d|5\d|6[0-7]):")
_BLOCK = re.compile(r"^(\.LBB\d+_\d+):(.*)$")
_FALL = re.compile(r"^; %bb\.\d+:(.*)$")


def check_assembly(text: str) -> int:
    """Returns the number of stream loops checked; raises on a violation."""
    lines = text.split("\n")
    member = []
    cur = None
    for line in lines:
        m = _BLOCK.match(line)
        rest = m.group(2) if m else (_FALL.match(line).group(1) if _FALL.match(line) else None)
        if rest is not None:
            inner = re.search(r"in Loop: Header=(BB\d+_\d+) Depth=1", rest)
            if inner:
                cur = inner.group(1)
            elif "Loop Header: Depth=1" in rest and m:
                cur = m.group(1)[2:]
            elif "Depth=2" in rest or "Parent Loop" in rest:
                pass  # a nested loop belongs to the loop around it
            else:
                cur = None
        member.append(cur)
    loops = {member[i] for i, line in enumerate(lines)
             if "s_load_dwordx16 s[36:51]" in line and "0x80" in line and member[i]}
    if not loops:
        raise RuntimeError("no stream loop found: the check no longer matches the kernel")
    for loop in loops:
        in_asm = False
        for i, line in enumerate(lines):
            if "ASMSTART" in line:
                in_asm = True
            elif "ASMEND" in line:
                in_asm = False
            elif member[i] == loop and not in_asm and not line.lstrip().startswith(";") and _PINNED.search(line):
                raise RuntimeError(f"pinned stream register touched outside the evaluation statements "
                                   f"(loop {loop}, line {i + 1}): {line.strip()}")
    return len(loops)


def check(hipcc: str, flags: list[str], source: str, out_dir: str) -> int:
    asm = os.path.join(out_dir, "forest_kernels_ranklds.s")
    subprocess.run([hipcc, *flags, "-x", "hip", "-S", "--cuda-device-only", source, "-o", asm], check=True,
                   stderr=subprocess.DEVNULL)
    with open(asm) as fh:
        return check_assembly(fh.read())


if __name__ == "__main__":
    print(check_assembly(open(sys.argv[1]).read()), "stream loops clean")
