"""Build-time check of the scorer's compiled code.

score_mlp.hip issues its operand loads (A fragments, B fragments, the block's constants) as
inline assembly and waits for them with hand-counted `s_waitcnt` instructions, because the
compiler's own counts cannot see the load-to-LDS operations that share the queue.  The price:
to the compiler such a load has written its destination register when it is *issued*, so
nothing stops it from copying, spilling or re-using that register before the data has
arrived.  This module walks the generated assembly and reports every instruction that touches
a vector register while a load into it can still be outstanding by the wait instructions seen
so far.  `build.py` runs it on every build and fails the build on a finding.

The walk is linear (program order as laid out, branches ignored) and models the two in-order
queues of a wavefront: vector memory (`vmcnt`) and LDS/scalar memory (`lgkmcnt`).  Because the
two arms of a branch are laid out one after the other, loads of the first arm still count as
outstanding in the second: a finding there can be a false one (it was, for a configuration
that is not built).  Following the branches instead does not help as it stands: the kernel
decides the parity of its K-tile count twice (which register set gets tile 0; whether one tile
runs ahead of the pair loop), and a walk over all paths takes the two impossible combinations
as well and reports their mismatched counts.  A finding stops the build so that the listing
gets read."""
from __future__ import annotations

import re
from typing import List, Set, Tuple

_LABEL = re.compile(r"^[.\w$]+:")


def _regs(token: str) -> Set[int]:
    token = token.strip().rstrip(",")
    m = re.match(r"^v\[(\d+):(\d+)\]$", token)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"^v(\d+)$", token)
    if m:
        return {int(m.group(1))}
    return set()


def _trim(queue: list, allowed: int) -> list:
    """State of an in-order queue after `s_waitcnt <counter>(allowed)`."""
    if allowed <= 0:
        return []
    return queue[-allowed:] if allowed < len(queue) else queue


def lint_kernel(lines: List[str]) -> List[Tuple[int, str]]:
    """`lines`: one kernel's instructions.  Returns (index, instruction) of every instruction
    that reads or writes a VGPR that an earlier load may not have written yet."""
    vm: List[Set[int]] = []      # outstanding vector-memory operations (destination registers)
    lgkm: List[Set[int]] = []    # outstanding LDS / scalar-memory operations
    found = []
    for i, raw in enumerate(lines):
        line = raw.split(";")[0].strip()
        if not line or line.startswith(".") or _LABEL.match(line):
            continue
        op, _, rest = line.partition(" ")
        toks = [t for t in re.split(r",\s*|\s+", rest) if t]
        if op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", rest)
            if m:
                vm = _trim(vm, int(m.group(1)))
            m = re.search(r"lgkmcnt\((\d+)\)", rest)
            if m:
                lgkm = _trim(lgkm, int(m.group(1)))
            if re.fullmatch(r"\s*0\s*", rest):      # s_waitcnt 0: everything
                vm, lgkm = [], []
            continue
        used = set().union(*[_regs(t) for t in toks]) if toks else set()
        in_flight = set().union(*vm, *lgkm) if (vm or lgkm) else set()
        is_load = re.match(r"^(global|buffer|flat|scratch)_load", op) is not None
        is_vm_other = re.match(r"^(global|buffer|flat|scratch)_(store|atomic)", op) is not None
        if is_load:
            # (a second load into a register that is still outstanding is not a finding: the two
            # arms of a branch are laid out one after the other, and loads return in order)
            dest = set() if "_lds_" in op else _regs(toks[0])
            if (used - dest) & in_flight:
                found.append((i, line))
            vm.append(dest)
        elif is_vm_other:
            if used & in_flight:
                found.append((i, line))
            vm.append(set())
        elif re.match(r"^ds_(read|load)", op):
            dest = _regs(toks[0])
            if (used - dest) & in_flight:
                found.append((i, line))
            lgkm.append(dest)
        elif op.startswith("ds_"):
            if used & in_flight:
                found.append((i, line))
            lgkm.append(set())
        elif re.match(r"^s_(buffer_)?load", op):
            lgkm.append(set())
        elif used & in_flight:
            found.append((i, line))
    return found


def split_kernels(asm_text: str, name_contains: str):
    """(symbol, instruction lines) of every function whose symbol contains `name_contains`."""
    lines = asm_text.split("\n")
    out = []
    i = 0
    while i < len(lines):
        m = re.match(r"^([\w$.]+):\s*;\s*@", lines[i])
        if m and name_contains in m.group(1):
            j = i + 1
            while j < len(lines) and not lines[j].startswith(".Lfunc_end"):
                j += 1
            out.append((m.group(1), lines[i + 1:j]))
            i = j
        i += 1
    return out


def lint_scorer_asm(asm_text: str, name_contains: str = "score_mlp_frag_kernel"):
    """{symbol: findings} for the scorer's kernels in a device assembly listing."""
    kernels = split_kernels(asm_text, name_contains)
    if not kernels:
        raise RuntimeError(f"no function matching {name_contains!r} in the assembly")
    return {sym: lint_kernel(body) for sym, body in kernels}
