"""Static check of the compiled kernels that issue LDS reads from inline assembly.

The compiler does not know that such a read is still in flight after the statement, so nothing
but the kernel's own wait (an assembly statement that takes the same registers as operands) may
touch a destination register in between: a copy made earlier would hold stale data, and a
register handed to other code would be overwritten when the LDS data arrives.

LDS operations of a wavefront complete in order, and `s_waitcnt lgkmcnt(N)` returns when at most N
of them are outstanding.  The scan keeps the queue of LDS operations in program order, retires all
but the youngest N at such a wait, and reports any instruction that names a destination register of
a read still in the queue, and any read whose address register is itself still pending.  Scalar
memory loads share the counter but return out of order: a wait for N > 0 never retires one of them,
and retires all LDS operations but the youngest N (at most N operations of any kind are outstanding
after it, and the outstanding LDS operations are always the youngest ones).

Second check, for MFMAs issued from assembly (the compiler inserts the wait states for its own): a matrix
instruction's result may be named by another kind of instruction only a number of wait states after the MFMA
was issued (its passes + 3; an instruction is one wait state, `s_nop N` is N + 1).  The next MFMA accumulating into the very same
registers is the one exception the hardware allows.  And the other way round: an MFMA may read a vector register
only two wait states after a vector instruction wrote it."""
import re

_READ = re.compile(r"(ds_read\w*|ds_load\w*) (v\[(\d+):(\d+)\]|v(\d+)), v(\d+)")


def _settle(op):
    """Wait states after the issue of this MFMA before another kind of instruction may name its result: the
    instruction's passes + 3 (what the compiler leaves after its own: 11 for the 8-pass 32x32x16, 7 for the 4-pass
    16x16x32 of the 16-bit formats)."""
    return 7 if "_16x16x" in op else 11


_AREG = re.compile(r"\ba\[(\d+):(\d+)\]|\ba(\d+)\b")


def _aregs(line):
    regs = set()
    for a, b, c in _AREG.findall(line):
        if a:
            regs.update(range(int(a), int(b) + 1))
        else:
            regs.add(int(c))
    return regs


def _regs(line):
    regs = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", line):
        regs.update(range(int(a), int(b) + 1))
    for a in re.findall(r"\bv(\d+)\b", line):
        regs.add(int(a))
    return regs


def scan(asm_text: str):
    """Returns {function: [(line number, instruction), ...]} of hazards.

    Every path through a function's branches is walked (a conditional branch forks the walk, an unconditional one
    is followed); a block is entered again for a new state of the queue it is reached with (up to four), so a
    read issued late in one loop iteration and used early in the next is seen."""
    lines = asm_text.split("\n")
    issues = {}
    # function boundaries
    starts = [(i, re.match(r"^(_Z\w+):", l).group(1)) for i, l in enumerate(lines) if re.match(r"^(_Z\w+):", l)]
    for k, (begin, fn) in enumerate(starts):
        end = starts[k + 1][0] if k + 1 < len(starts) else len(lines)
        labels = {}
        for i in range(begin, end):
            m = re.match(r"^(\.LBB\w+):", lines[i])
            if m:
                labels[m.group(1)] = i
        found = []

        def report(i, text):
            if (i, text) not in found:
                found.append((i, text))

        seen, visits = set(), {}   # a label is entered with at most four different queue states
        work = [(begin + 1, ())]
        while work:
            i, q = work.pop()
            queue = [None if e is None else set(e) for e in q]

            def pending():
                out = set()
                for e in queue:
                    if e:
                        out |= e
                return out

            recent = []   # [vector registers, accumulator registers, wait states since issue] of the latest MFMAs
            valu = []     # (vector registers written, wait states since) of the latest vector instructions
            while i < end:
                raw = lines[i]
                line = raw.strip()
                if line and line[0] not in ";." and not re.match(r"^(\.LBB\w+):", raw):
                    vr, ar = _regs(line), _aregs(line)
                    if line.startswith("v_mfma") or line.startswith("v_smfma"):
                        ops = [o.strip() for o in line.split(None, 1)[1].split(",")]
                        if any(age < 2 and (regs & _regs(",".join(ops[1:]))) for regs, age in valu):
                            report(i, line)
                        dst_v, dst_a = _regs(ops[0]), _aregs(ops[0])
                        for e in recent:
                            same = e[0] == dst_v and e[1] == dst_a and ops[3].split()[0] == ops[0]
                            src = ",".join(ops[1:3]) + ("" if same else "," + ops[3])
                            if e[2] < e[3] and ((_regs(src) & e[0]) or (_aregs(src) & e[1]) or
                                                       (not same and ((dst_v & e[0]) or (dst_a & e[1])))):
                                report(i, line)
                        recent = [e for e in recent if not (e[0] == dst_v and e[1] == dst_a)]
                        recent.append([dst_v, dst_a, 0, _settle(line.split()[0])])
                    else:
                        for e in recent:
                            if e[2] < e[3] and ((vr & e[0]) or (ar & e[1])):
                                report(i, line)
                    m = re.match(r"s_nop (\d+)", line)
                    step = int(m.group(1)) + 1 if m else 1
                    valu = [(regs, age + step) for regs, age in valu if age + step < 2]
                    if line.startswith("v_") and not line.startswith("v_mfma") and not line.startswith("v_smfma") \
                            and not line.startswith("v_accvgpr_read") and not line.startswith("v_cmp"):
                        valu.append((_regs(line.split(None, 1)[1].split(",")[0]), 0))
                    for e in recent:
                        e[2] += step
                    recent = [e for e in recent if e[2] < e[3]]
                if re.match(r"^(\.LBB\w+):", raw):
                    key = (i, tuple(None if e is None else frozenset(e) for e in queue))
                    if key in seen or visits.get(i, 0) >= 4:
                        break
                    seen.add(key)
                    visits[i] = visits.get(i, 0) + 1
                    i += 1
                    continue
                if not line or line[0] in ";.":
                    i += 1
                    continue
                m = _READ.match(line)
                if m:
                    if int(m.group(6)) in pending():
                        report(i, line)
                    dst = set(range(int(m.group(3)), int(m.group(4)) + 1)) if m.group(3) else {int(m.group(5))}
                    # a read into registers that an older read still owns would race with it
                    if dst & pending():
                        report(i, line)
                    queue.append(dst)
                    i += 1
                    continue
                if line.startswith("ds_"):
                    if _regs(line) & pending():
                        report(i, line)
                    queue.append(set())
                    i += 1
                    continue
                if re.match(r"s_(buffer_)?load_", line) or line.startswith("s_memtime") or line.startswith("s_memrealtime"):
                    queue.append(None)
                    i += 1
                    continue
                if line.startswith("s_waitcnt"):
                    m = re.search(r"lgkmcnt\((\d+)\)", line)
                    if m:
                        n = int(m.group(1))
                        if n == 0:
                            queue = []
                        else:
                            # at most n operations are outstanding, and the outstanding LDS operations are the
                            # youngest ones: all LDS entries but the youngest n are done, whatever the scalar
                            # loads did
                            lds = [k2 for k2, e in enumerate(queue) if e is not None]
                            done = set(lds[:max(0, len(lds) - n)])
                            queue = [e for k2, e in enumerate(queue) if k2 not in done]
                    i += 1
                    continue
                if line.startswith("s_endpgm"):
                    break   # reads still in flight here touch no live register (paths that skip their use end so)
                m = re.match(r"s_cbranch_\w+ (\.LBB\w+)", line)
                if m:
                    if m.group(1) in labels:
                        work.append((labels[m.group(1)], tuple(None if e is None else frozenset(e) for e in queue)))
                    i += 1
                    continue
                m = re.match(r"s_branch (\.LBB\w+)", line)
                if m:
                    if m.group(1) in labels:
                        i = labels[m.group(1)]
                        continue
                    break
                if not line.startswith("s_"):
                    if _regs(line) & pending():
                        report(i, line)
                i += 1
        if found:
            issues[fn] = sorted(found)
    return issues
