"""Build-time check for the kernels whose MFMAs are asm statements (the persistent GEMM).

The compiler inserts the wait states an MFMA needs around instructions it recognises; an MFMA written as an asm
statement is opaque to it.  The kernel keeps its accumulators where they are and separates the K loop from the code
that reads or clears them with explicit s_nop, but the register allocator is free to move an accumulator (through
v_accvgpr_read / _write / _mov) anywhere between two asm statements.  This script reads the compiler's assembly
listing of the kernel source (produced by the build with -S; nothing is disassembled) and fails if, in a kernel
named on the command line,

  * an instruction other than an MFMA touches an AGPR that an MFMA wrote fewer than MFMA_TO_OTHER wait states
    before it, or
  * an MFMA reads or overwrites an AGPR that another instruction wrote fewer than OTHER_TO_MFMA wait states before,

following straight-line order and every branch (the instructions before a branch against those after its target).
Every instruction counts as one wait state, `s_nop n` as n + 1.  The distances are those of the longest MFMA
(16 passes) in the CDNA3 instruction set manual's table of required software wait states, so they cover the
4-pass MFMA used here with room to spare.

    python check_mfma_hazards.py listing.s gemm_p256_kernel
"""
import re
import sys

MFMA_TO_OTHER = 19
OTHER_TO_MFMA = 4
WINDOW = max(MFMA_TO_OTHER, OTHER_TO_MFMA)

AREG = re.compile(r"\ba(\d+)\b|\ba\[(\d+):(\d+)\]")


def aregs(text):
    regs = set()
    for m in AREG.finditer(text):
        if m.group(1) is not None:
            regs.add(int(m.group(1)))
        else:
            regs.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return regs


def parse_kernel(lines):
    """-> list of (wait_state_index, kind, reads, writes, text), labels {name: position in list}, branches [(pos, target)]"""
    ins, labels, branches = [], {}, []
    t = 0
    for raw in lines:
        line = raw.split(";")[0].strip()
        if not line:
            continue
        m = re.match(r"^(\.LBB\d+_\d+):", line)
        if m:
            labels[m.group(1)] = len(ins)
            continue
        if line.startswith(".") or line.endswith(":"):
            continue
        op, _, rest = line.partition(" ")
        ops = [o.strip() for o in rest.split(",")]
        if op.startswith("v_mfma"):
            dst, src_c = aregs(ops[0]), aregs(ops[3]) if len(ops) > 3 else set()
            ins.append((t, "mfma", dst | src_c, dst, line))
        else:
            touched = aregs(rest)
            if op.startswith("v_accvgpr_read"):
                reads, writes = aregs(ops[1]), set()
            elif op.startswith("v_accvgpr_write"):
                reads, writes = set(), aregs(ops[0])
            elif op.startswith("v_accvgpr_mov"):
                reads, writes = aregs(ops[1]), aregs(ops[0])
            else:
                reads, writes = touched, touched       # anything else that names an AGPR: assume both
            ins.append((t, "other", reads, writes, line))
            m = re.match(r"s_(cbranch\w*|branch)$", op)
            if m and ops and ops[0].startswith(".LBB"):
                branches.append((len(ins) - 1, ops[0]))
        n = re.match(r"s_nop\s+(\d+)", line)
        t += int(n.group(1)) + 1 if n else 1
    return ins, labels, branches


def check_pairs(before, after, shift, problems, where):
    """Every instruction of `before` against every instruction of `after`; an instruction of `after` at time ta is
    issued ta + shift - tb wait states after one of `before` at time tb (shift = 0 along straight-line code)."""
    for tb, kb, rb, wb, xb in before:
        for ta, ka, ra, wa, xa in after:
            dist = ta + shift - tb
            if kb == "mfma" and ka == "other" and dist < MFMA_TO_OTHER and wb & (ra | wa):
                problems.append("%s: %d wait states between\n    %s\n    %s" % (where, dist, xb, xa))
            if kb == "other" and ka == "mfma" and dist < OTHER_TO_MFMA and wb & ra:
                problems.append("%s: %d wait states between\n    %s\n    %s" % (where, dist, xb, xa))


def check_kernel(name, lines):
    ins, labels, branches = parse_kernel(lines)
    problems = []
    # straight-line order: every instruction against the WINDOW wait states before it
    for i, cur in enumerate(ins):
        j = i - 1
        prev = []
        while j >= 0 and cur[0] - ins[j][0] <= WINDOW:
            prev.append(ins[j])
            j -= 1
        check_pairs(prev, [cur], 0, problems, name)
    # every branch: the instructions up to it against the instructions from its target on, as if the target followed
    # the branch directly
    for pos, target in branches:
        if target not in labels or labels[target] >= len(ins):
            continue
        t_branch = ins[pos][0]
        tail = [x for x in ins[max(0, pos - WINDOW):pos + 1] if t_branch - x[0] <= WINDOW]
        h0 = labels[target]
        head = [x for x in ins[h0:h0 + WINDOW + 1] if x[0] - ins[h0][0] <= WINDOW]
        check_pairs(tail, head, t_branch + 1 - ins[h0][0], problems, "%s (branch to %s)" % (name, target))
    n_mfma = sum(1 for x in ins if x[1] == "mfma")
    return n_mfma, problems


def main(argv):
    if len(argv) != 3:
        sys.exit(__doc__)
    text = open(argv[1]).read().split("\n")
    pattern = argv[2]
    starts = [i for i, l in enumerate(text) if re.match(r"^_Z\w*%s\w*:" % re.escape(pattern), l)]
    if not starts:
        sys.exit("check_mfma_hazards: no kernel matching %r in %s" % (pattern, argv[1]))
    bad = 0
    for s in starts:
        e = s
        while e < len(text) and ".end_amdhsa_kernel" not in text[e] and not text[e].startswith("\t.section\t.rodata"):
            e += 1
        name = text[s].split(":")[0]
        n_mfma, problems = check_kernel(name, text[s + 1:e])
        print("check_mfma_hazards: %s: %d MFMAs, %d problem(s)" % (name, n_mfma, len(problems)))
        for p in problems[:20]:
            print("  " + p)
        bad += len(problems)
    sys.exit(1 if bad else 0)


if __name__ == "__main__":
    main(sys.argv)
