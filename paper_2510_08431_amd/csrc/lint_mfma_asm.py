"""Build-time check of the hand-written MFMA statements in the compiled gfx950 assembly.

The sweep kernel issues its score products as inline assembly (destination in arithmetic registers).  The
compiler schedules and allocates registers around such statements but does not know what is inside them, so it
inserts none of the wait states the hardware needs around an MFMA.  The kernel provides them itself; this check
reads the assembly the compiler produced and fails the build if an instruction the compiler placed (a register
copy after allocation, say) ended up inside one of those windows.  Rules, for 8-pass MFMAs on gfx950, in wait
states (one per issued instruction, N + 1 for `s_nop N`):

  R1  a vector-ALU instruction that writes a register an assembly MFMA reads (A, B or C operand) must be at least
      2 wait states before it;
  R2  after an assembly MFMA, no instruction other than an MFMA accumulating into exactly the same registers may
      read or write its destination registers for 11 wait states.

Both are checked along straight-line code; a label or branch ends the window of R1 (nothing is known about the
other path) and R2 keeps scanning through fall-through labels.  Usage: python lint_mfma_asm.py file.s [...]
"""
import re
import sys

VALU_WRITE_TO_MFMA_READ = 2
MFMA8_WRITE_TO_OTHER_ACCESS = 11

_REG = re.compile(r"\b([va])(?:\[(\d+):(\d+)\]|(\d+)\b)")


def regs_of(operand_text):
    """Set of (file, index) registers named in a piece of operand text ('v[4:7]', 'a12', 'v3')."""
    out = set()
    for m in _REG.finditer(operand_text):
        f = m.group(1)
        if m.group(4) is not None:
            out.add((f, int(m.group(4))))
        else:
            out.update((f, i) for i in range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def split_operands(line):
    parts = line.split(None, 1)
    if len(parts) < 2:
        return parts[0], []
    return parts[0], [p.strip() for p in parts[1].split(",")]


def wait_states(op, operands):
    if op == "s_nop":
        return int(operands[0], 0) + 1
    return 1


def writes_reads(op, operands):
    """(registers written, registers read) of an ordinary instruction, conservatively: the first operand of a
    vector or LDS/memory-load instruction is its destination, everything else is read; stores read everything."""
    if not operands:
        return set(), set()
    stores = op.startswith(("ds_write", "ds_store", "global_store", "buffer_store", "flat_store", "scratch_store",
                            "global_load_lds", "s_"))
    if stores:
        return set(), set().union(*(regs_of(o) for o in operands))
    first = regs_of(operands[0])
    rest = set().union(*(regs_of(o) for o in operands[1:])) if len(operands) > 1 else set()
    if op.startswith(("v_cmp", "v_cmpx")):          # compares write a scalar/VCC; every vector operand is read
        return set(), first | rest
    if op.startswith(("v_fmac", "v_mac", "v_dot2c", "v_pk_fmac")):   # destination is also an addend
        rest |= first
    return first, rest


def lint(text, name="<asm>"):
    """Returns a list of violation strings for one assembly file."""
    lines = text.split("\n")
    insns = []      # (line_no, op, operands, in_asm, is_label_or_branch)
    in_asm = False
    for no, raw in enumerate(lines, 1):
        l = raw.strip()
        if l.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if l.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not l or l.startswith((";", "//", ".")) and not re.match(r"^\.L\w+:", l):
            continue
        if re.match(r"^[\w.$]+:", l):
            insns.append((no, "<label>", [], False, True))
            continue
        l = l.split(";")[0].strip()
        if not l:
            continue
        op, operands = split_operands(l)
        insns.append((no, op, operands, in_asm, op.startswith(("s_cbranch", "s_branch", "s_endpgm", "s_setpc"))))

    problems = []
    for i, (no, op, operands, asm, _) in enumerate(insns):
        if not (asm and op.startswith("v_mfma")):
            continue
        dst = regs_of(operands[0])
        srcs = set().union(*(regs_of(o) for o in operands[1:4]))
        # R1: look back
        ws, j = 0, i - 1
        while j >= 0 and ws < VALU_WRITE_TO_MFMA_READ:
            pno, pop, pops, pasm, pbar = insns[j]
            if pbar:
                break
            if pop.startswith("v_") and not pop.startswith("v_mfma"):
                w, _ = writes_reads(pop, pops)
                if w & srcs:
                    problems.append(f"{name}:{no}: {op} reads {sorted(w & srcs)[:4]} written by {pop} (line {pno}) "
                                    f"only {ws} wait state(s) earlier (need {VALU_WRITE_TO_MFMA_READ})")
            ws += wait_states(pop, pops)
            j -= 1
        # R2: look ahead
        ws, j = 0, i + 1
        while j < len(insns) and ws < MFMA8_WRITE_TO_OTHER_ACCESS:
            nno, nop, nops, nasm, nbar = insns[j]
            if nop == "<label>":
                j += 1
                continue
            if nbar:
                break
            if nop.startswith("v_mfma"):
                ndst = regs_of(nops[0])
                nsrc_ab = set().union(*(regs_of(o) for o in nops[1:3]))
                nsrc_c = regs_of(nops[3]) if len(nops) > 3 else set()
                chain = ndst == dst and (nsrc_c == dst or not nsrc_c)
                touched = (nsrc_ab & dst) | (set() if chain else ((ndst | nsrc_c) & dst))
            else:
                w, r = writes_reads(nop, nops)
                touched = (w | r) & dst
            if touched:
                problems.append(f"{name}:{nno}: {nop} touches {sorted(touched)[:4]}, destination of the assembly {op} at "
                                f"line {no}, after {ws} wait state(s) (need {MFMA8_WRITE_TO_OTHER_ACCESS})")
            ws += wait_states(nop, nops)
            j += 1
    return problems


def count_asm_mfma(text):
    n, in_asm = 0, False
    for raw in text.split("\n"):
        l = raw.strip()
        if l.startswith(";;#ASMSTART"):
            in_asm = True
        elif l.startswith(";;#ASMEND"):
            in_asm = False
        elif in_asm and l.startswith("v_mfma"):
            n += 1
    return n


def main(argv):
    bad = 0
    for path in argv:
        with open(path) as f:
            text = f.read()
        problems = lint(text, path)
        print(f"{path}: {count_asm_mfma(text)} assembly MFMAs checked, {len(problems)} problem(s)")
        for p in problems[:20]:
            print("  " + p)
        bad += len(problems)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
