"""Build-time guard over the compiler's gfx950 assembly of the matrix-core kernels.

v_mfma ignores the execution mask.  The compiler lowers a branch on a value it cannot prove
wave-uniform to an exec-mask update, and for short blocks it drops the branch that would skip the
block when the mask is empty; a matrix instruction in such a block then runs on registers whose loads
were skipped.  The kernels keep every condition around a matrix instruction scalar; this scan checks
the result: it fails when a v_mfma sits between a saveexec that no skip branch follows and the
restore of exec.
"""
from __future__ import annotations

import re
from typing import List

_LABEL = re.compile(r"^(_Z\w+):")


def scan(asm_text: str) -> List[str]:
    """Returns one message per suspect matrix instruction."""
    out: List[str] = []
    kernel = "?"
    pending = 0   # line of a saveexec whose next instruction has not been seen yet
    masked = 0    # line of the saveexec that opened an unskipped masked block
    for ln, line in enumerate(asm_text.splitlines(), 1):
        t = line.strip()
        m = _LABEL.match(t)
        if m:
            kernel, pending, masked = m.group(1), 0, 0
            continue
        if not t or t[0] in ";.":
            continue
        fields = t.replace(",", " ").split()
        ins = fields[0]
        if pending:
            if not ins.startswith("s_cbranch_exec"):
                masked = pending
            pending = 0
        if "saveexec" in ins:
            pending = ln
            continue
        if ins in ("s_or_b64", "s_mov_b64") and len(fields) > 1 and fields[1] == "exec":
            masked = 0
        if ins.startswith("v_mfma") and masked:
            out.append(f"line {ln}: {kernel}: matrix instruction in a masked block without a skip branch "
                       f"(exec narrowed at line {masked})")
    return out
