"""Static check of the generated gfx950 code, run by the build.

decode_mfma.hip requests a wavefront's query rows with ``global_load_dwordx4`` written as inline
assembly with register outputs and waits for them later by count (the tile loads requested after
them must stay in flight, which a compiler-placed wait would not allow).  Between such a load and
the wait the hardware still owes the register its value: an instruction that reads the register
there sees stale data, one that writes it is overwritten when the load lands, and if the compiler
had moved an address into it the next access would go anywhere.  Nothing in the language forbids
the compiler to do that, so the build looks at what it actually did and fails if any pending
destination register is named by another instruction before the next ``s_waitcnt`` on ``vmcnt``.
"""
from __future__ import annotations

import re
from typing import Dict, List, Set, Tuple

_LOAD = re.compile(r"global_load_dwordx4 v\[(\d+):(\d+)\], v\[(\d+):(\d+)\], off")
_VREG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
_LABEL = re.compile(r"^(_Z\S+):")


def _regs(m) -> Set[int]:
    return {int(m.group(1))} if m.group(1) else set(range(int(m.group(2)), int(m.group(3)) + 1))


def kernels(asm: str) -> Dict[str, List[str]]:
    """Function name -> its lines (comments stripped), for every global symbol of the listing."""
    lines = asm.split("\n")
    starts = [(i, _LABEL.match(l).group(1)) for i, l in enumerate(lines) if _LABEL.match(l)]
    out = {}
    for k, (s0, name) in enumerate(starts):
        e0 = starts[k + 1][0] if k + 1 < len(starts) else len(lines)
        out[name] = [l.split(";")[0] for l in lines[s0 + 1:e0]]
    return out


def pending_register_violations(body: List[str]) -> Tuple[int, List[str]]:
    """(number of loads with register outputs, offending instructions).  The listing is walked in
    program order: a load's destination registers are pending until the next wait on the vector
    memory counter; until then no other instruction may name them, and no later load may take its
    address from them."""
    pending: Set[int] = set()
    loads, bad = 0, []
    for l in body:
        m = _LOAD.search(l)
        if m:
            loads += 1
            if set(range(int(m.group(3)), int(m.group(4)) + 1)) & pending:
                bad.append(l.strip())
            pending |= set(range(int(m.group(1)), int(m.group(2)) + 1))
            continue
        if "s_waitcnt" in l and "vmcnt" in l:
            pending.clear()
            continue
        if pending:
            for r in _VREG.finditer(l):
                if _regs(r) & pending:
                    bad.append(l.strip())
                    break
    return loads, bad


def check_listing(asm: str, name_filter: str) -> Dict[str, int]:
    """Raises RuntimeError if a kernel whose name contains name_filter touches a pending register;
    returns kernel name -> number of such loads it holds."""
    seen = {}
    for name, body in kernels(asm).items():
        if name_filter not in name:
            continue
        n, bad = pending_register_violations(body)
        if bad:
            raise RuntimeError(f"{name}: registers still owed to a load are used before the wait:\n  " + "\n  ".join(bad[:8]))
        seen[name] = n
    return seen
