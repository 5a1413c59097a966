"""Build-time check of the device assembly of the sources whose kernels issue global loads by hand.

A load written in inline asm (`global_load_dwordx4 v[a:b], ...`) returns at once; its destination
registers hold the data only after an `s_waitcnt vmcnt(N)` that the load is old enough for.  Until then
no instruction may read or write them: a copy would take the old contents, and an overwritten register
would be overwritten again when the data lands.  The kernels keep that rule in their source (every
register filled by such a load passes through an await_*() before its first use), but the compiler is
free to move or copy a variable between the two asm statements - it cannot know the register is not
ready - and it does so where a loop closes with the variable in another register than it opened with.

The check follows every path of a kernel's control-flow graph.  State = the registers that may still be
in flight, each with the least number of vector-memory loads issued after it on any path (loads return
in order, so `s_waitcnt vmcnt(N)` retires exactly the entries with at least N younger loads; stores are
not counted as younger: they may complete out of order with loads, so counting them would be
optimistic).  Every instruction that names an in-flight register and is neither the wait that retires it
nor a later load into it is reported.  Waits and loads of the compiler's own count like the hand-written
ones: the hardware does not tell them apart.
"""
import re

_LABEL = re.compile(r"^([.\w$]+):")
_BRANCH = re.compile(r"^(s_cbranch_\w+|s_branch)\s+([.\w$]+)")
_VRANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_VONE = re.compile(r"\bv(\d+)\b")
_VMCNT = re.compile(r"vmcnt\((\d+)\)")
_CAP = 64   # the counter has six bits: nothing is ever younger than that


def _vregs(text):
    out = set()
    for a, b in _VRANGE.findall(text):
        out.update(range(int(a), int(b) + 1))
    out.update(int(a) for a in _VONE.findall(text))
    return out


def _is_vmem_load(t):
    op = t.split()[0]
    return op.startswith(("global_load", "buffer_load", "flat_load", "scratch_load")) or \
        (op.startswith(("global_atomic", "buffer_atomic", "flat_atomic")) and " glc" in t)


class _Ins:
    __slots__ = ("line", "text", "hand")

    def __init__(self, line, text, hand):
        self.line, self.text, self.hand = line, text, hand


def _functions(asm_text):
    """(name, [(line number, text, inside inline asm) | label]) for every function of the file."""
    funcs, cur, name, in_asm = [], None, None, False
    types = set(re.findall(r"\.type\s+([.\w$]+),@function", asm_text))
    for i, raw in enumerate(asm_text.split("\n"), 1):
        t = raw.split(";")[0].strip() if not raw.strip().startswith(";;#") else raw.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t:
            continue
        m = _LABEL.match(t)
        if m:
            if m.group(1) in types:
                name, cur = m.group(1), []
                funcs.append((name, cur))
            elif cur is not None:
                cur.append(m.group(1))
            continue
        if t.startswith("."):
            if t.startswith(".Lfunc_end") or t.startswith(".section") or t.startswith(".size"):
                cur = None if t.startswith((".size", ".section")) else cur
            continue
        if cur is not None:
            cur.append(_Ins(i, t, in_asm))
    return funcs


def _blocks(items):
    """Basic blocks: list of (labels, instructions, successor labels, falls through)."""
    blocks, labels, ins = [], [], []

    def close(succ, fall):
        nonlocal labels, ins
        if labels or ins:
            blocks.append((labels, ins, succ, fall))
        labels, ins = [], []

    for it in items:
        if isinstance(it, str):
            if ins:
                close([], True)
            labels.append(it)
            continue
        ins.append(it)
        m = _BRANCH.match(it.text)
        if m:
            close([m.group(2)], m.group(1) != "s_branch")
        elif it.text.startswith(("s_endpgm", "s_setpc", "s_trap")):
            close([], False)
    close([], False)
    return blocks


def _step(state, it, report):
    """Advance `state` (register -> (younger loads, line of the load)) over one instruction."""
    t = it.text
    if t.startswith("s_waitcnt"):
        m = _VMCNT.search(t)
        if m:
            n = int(m.group(1))
            for r in [r for r, (y, _) in state.items() if y >= n]:
                del state[r]
        return
    regs = _vregs(t)
    if _is_vmem_load(t):
        dst = _vregs(t.split(",")[0]) if "_lds_" not in t.split()[0] else set()
        hit = (regs - dst) & state.keys()   # an address taken from a register in flight
        if hit and report is not None:
            report(it, hit, state)
        for r in state:
            y, ln = state[r]
            state[r] = (min(y + 1, _CAP), ln)
        if it.hand:
            for r in dst:
                state[r] = (0, it.line)
        else:
            for r in dst:          # the compiler's own load: it waits for it itself
                state.pop(r, None)
        return
    hit = regs & state.keys()
    if hit and report is not None:
        report(it, hit, state)


def check_hand_issued_loads(asm_text, name):
    """Raise RuntimeError when a path through a kernel of `asm_text` touches the destination of a
    hand-issued load before a wait has retired it."""
    bad = []
    for fname, items in _functions(asm_text):
        blocks = _blocks(items)
        index = {}
        for b, (labels, _, _, _) in enumerate(blocks):
            for lab in labels:
                index[lab] = b
        succs = []
        for b, (_, _, targets, fall) in enumerate(blocks):
            s = [index[x] for x in targets if x in index]
            if fall and b + 1 < len(blocks):
                s.append(b + 1)
            succs.append(s)
        entry = [None] * len(blocks)
        entry[0] = {}
        work = [0]
        while work:
            b = work.pop()
            state = dict(entry[b])
            for it in blocks[b][1]:
                _step(state, it, None)
            for s in succs[b]:
                if entry[s] is None:
                    entry[s] = dict(state)
                    work.append(s)
                    continue
                changed = False
                for r, (y, ln) in state.items():
                    if r not in entry[s] or entry[s][r][0] > y:
                        entry[s][r] = (y, ln)
                        changed = True
                if changed:
                    work.append(s)
        for b, (_, ins, _, _) in enumerate(blocks):
            if entry[b] is None:
                continue
            state = dict(entry[b])

            def report(it, hit, st):
                r = min(hit)
                bad.append(f"{name}: {fname[:80]}: line {it.line}: `{it.text[:70]}` touches v{sorted(hit)[:8]}, "
                           f"loaded by hand at line {st[r][1]} with {st[r][0]} younger loads and no wait that covers it")

            for it in ins:
                _step(state, it, report)
    if bad:
        raise RuntimeError(f"{len(bad)} uses of registers whose hand-issued loads may still be in flight:\n  " + "\n  ".join(bad[:12]))
