"""A check of the compiled kernels' assembly (host logic, no GPU).

The dense kernels issue their LDS fragment reads from inline assembly and wait for them one pipeline step later.  The
compiler takes an assembly statement's results for present as soon as the statement is over, so it may place a register
copy (at a branch or a loop boundary) that reads or overwrites those registers before the wait - the copy then moves
whatever the registers held before.  `scan` walks the assembly of every kernel along fall-through paths and reports any
instruction that touches a register an assembly-issued LDS read is still filling."""
import re


def _regs(line):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", line):
        if m.group(1):
            out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def scan(asm_text, window=80):
    """Returns a list of (kernel, line number, instruction, line of the pending read)."""
    found = []
    kernel, pending, in_asm = None, {}, False
    for ln, raw in enumerate(asm_text.splitlines(), 1):
        t = raw.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        m = re.match(r"^(_Z\w+):", t)
        if m:
            kernel, pending = m.group(1), {}
            continue
        if not t or t.startswith(";") or t.startswith("."):
            continue
        op = t.split()[0]
        if op in ("s_branch", "s_endpgm", "s_setpc_b64"):
            pending = {}          # the next line is not reached by falling through
            continue
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", t)
            if m and int(m.group(1)) == 0:
                pending = {}
            continue
        pending = {r: l for r, l in pending.items() if ln - l < window}
        if in_asm and op.startswith("ds_read"):
            dst = _regs(t.split()[1].rstrip(","))
            hit = (_regs(t) - dst) & set(pending)
            if hit:
                found.append((kernel, ln, t, pending[min(hit)]))
            for r in dst:
                pending[r] = ln
            continue
        hit = _regs(t) & set(pending)
        if hit:
            found.append((kernel, ln, t, pending[min(hit)]))
    return found
