"""Static check of the device assembly of kernels that issue LDS reads by hand and wait for them by count.

Such a kernel names, with every "s_waitcnt lgkmcnt(N)" it writes, which of its outstanding LDS reads have
arrived.  The compiler knows nothing of that: between the read (an inline-asm statement whose output is a
register) and the wait (another one, tied to the same variable) its register allocator is free to copy the
variable into another register, and such a copy reads the register before the data is there.  The program is
then wrong only when the LDS answers late, so no test finds it reliably.  This check walks every path through a
kernel's instruction listing, keeps the queue of outstanding LDS operations with the registers they will write,
shortens it at each wait, and reports every instruction that touches a register whose read is still in flight.

LDS operations answer in order, so after "lgkmcnt(N)" at most the N youngest are outstanding.  Scalar memory
loads share the counter and answer out of order, but one that is outstanding only takes a place among the N:
the bound on the LDS operations holds with or without it, and the check leaves scalar loads out.
"""
import re
import sys

_LABEL = re.compile(r"^(\.LBB\d+_\d+):")
_FUNC = re.compile(r"^(_Z\w+):")
_VREG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
_LGKM = re.compile(r"lgkmcnt\((\d+)\)")


def _vregs(text):
    regs = set()
    for m in _VREG.finditer(text):
        if m.group(1) is not None:
            regs.add(int(m.group(1)))
        else:
            regs.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return regs


def _split_instruction(line):
    """-> (mnemonic, [operand texts]) of one instruction line, comments removed; None for anything else."""
    line = line.split(";", 1)[0].strip()
    if not line or line.startswith((".", "#")) or line.endswith(":"):
        return None
    parts = line.split(None, 1)
    ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
    # a register range contains no comma, modifiers (offset:.., op_sel..) ride on the last operand: harmless here
    return parts[0], ops


def kernel_bodies(asm_text, name_part):
    """{mangled name: [lines]} of the functions whose name contains name_part."""
    out, name, body = {}, None, []
    for line in asm_text.splitlines():
        m = _FUNC.match(line)
        if m:
            name, body = m.group(1), []
            continue
        if name is None:
            continue
        if line.startswith(".Lfunc_end"):
            if name_part in name:
                out[name] = body
            name = None
            continue
        body.append(line)
    return out


def check_kernel(lines):
    """-> list of (line index, text, registers) for every touch of a register with an LDS read in flight."""
    # basic blocks
    labels = {}
    instrs = []  # (mnemonic, operands, raw)
    for line in lines:
        m = _LABEL.match(line)
        if m:
            labels[m.group(1)] = len(instrs)
            continue
        ins = _split_instruction(line)
        if ins:
            instrs.append((ins[0], ins[1], line.strip()))
    problems = {}
    seen = set()
    heads = set(labels.values())

    def normal(queue):
        """Oldest entries that write no register cannot matter any more: dropping them keeps the set of
        states finite in loops that only write LDS."""
        i = 0
        while i < len(queue) and not queue[i]:
            i += 1
        return queue[i:][-16:]  # the counter holds 15

    work = [(0, ())]  # (instruction index, registers of the outstanding LDS operations oldest first)
    while work:
        pc, queue = work.pop()
        queue = list(queue)
        while pc < len(instrs):
            if pc in heads:
                key = (pc, tuple(queue))
                if key in seen:
                    break
                seen.add(key)
            mn, ops, raw = instrs[pc]
            pending = set().union(*queue) if queue else set()
            if mn == "s_waitcnt":
                m = _LGKM.search(raw)
                if m:
                    n = int(m.group(1))
                    if n < len(queue):
                        queue = queue[len(queue) - n:]
            elif mn.startswith("ds_"):
                reads = mn.startswith(("ds_read", "ds_bpermute", "ds_permute", "ds_swizzle")) or "_rtn" in mn
                dst = _vregs(ops[0]) if reads and ops else set()
                src = set()
                for o in (ops[1:] if reads else ops):
                    src |= _vregs(o)
                hit = src & pending
                if hit:
                    problems[pc] = (raw, sorted(hit))
                queue.append(frozenset(dst))
            else:
                hit = set()
                for o in ops:
                    hit |= _vregs(o) & pending
                if hit:
                    problems[pc] = (raw, sorted(hit))
                if mn == "s_endpgm":
                    break
                if mn == "s_branch":
                    queue = normal(queue)
                    pc = labels[ops[0]]
                    continue
                if mn.startswith("s_cbranch"):
                    queue = normal(queue)
                    work.append((labels[ops[0]], tuple(queue)))
            pc += 1
            if pc in heads:
                queue = normal(queue)
    return [(pc, raw, regs) for pc, (raw, regs) in sorted(problems.items())]


def check_text(asm_text, name_part):
    """Raise RuntimeError naming every offending instruction of every kernel whose name contains name_part."""
    bodies = kernel_bodies(asm_text, name_part)
    if not bodies:
        raise RuntimeError(f"no kernel named *{name_part}* in the assembly listing")
    bad = []
    for name, lines in bodies.items():
        for pc, raw, regs in check_kernel(lines):
            bad.append(f"{name}: instruction {pc}: '{raw}' touches v{regs} while its LDS read is in flight")
    if bad:
        raise RuntimeError("hand-scheduled LDS reads are used before their wait:\n" + "\n".join(bad[:40]))
    return len(bodies)


if __name__ == "__main__":
    with open(sys.argv[1]) as f:
        print(check_text(f.read(), sys.argv[2] if len(sys.argv) > 2 else "k_gemm_tile"), "kernels checked")
