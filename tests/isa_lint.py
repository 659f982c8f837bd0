"""Static check of the compiled kernels that issue LDS reads from inline assembly.

The compiler does not know that such a read is still in flight after the statement, so nothing
but the kernel's own wait (an assembly statement that takes the same registers as operands) may
touch a destination register in between: a copy made earlier would hold stale data, and a
register handed to other code would be overwritten when the LDS data arrives.

LDS operations of a wavefront complete in order, and `s_waitcnt lgkmcnt(N)` returns when at most N
of them are outstanding.  The scan keeps the queue of LDS operations in program order, retires all
but the youngest N at such a wait, and reports any instruction that names a destination register of
a read still in the queue, and any read whose address register is itself still pending.  Scalar
memory loads share the counter but return out of order: with one in the queue only a wait for zero
retires anything.  A loop is walked twice (the second time with the queue the first pass left), so a
read issued late in one iteration and used early in the next is seen."""
import re

_READ = re.compile(r"(ds_read\w*|ds_load\w*) (v\[(\d+):(\d+)\]|v(\d+)), v(\d+)")


def _regs(line):
    regs = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", line):
        regs.update(range(int(a), int(b) + 1))
    for a in re.findall(r"\bv(\d+)\b", line):
        regs.add(int(a))
    return regs


def scan(asm_text: str):
    """Returns {function: [(line number, instruction), ...]} of hazards."""
    lines = asm_text.split("\n")
    fn = None
    queue = []          # one entry per LDS / scalar-memory operation in flight: set of registers, or None for scalar memory
    issues = {}
    labels = {}
    rewalked = set()

    def pending():
        out = set()
        for e in queue:
            if e:
                out |= e
        return out

    def report(i, text):
        lst = issues.setdefault(fn, [])
        if (i, text) not in lst:
            lst.append((i, text))

    i = 0
    while i < len(lines):
        raw = lines[i]
        line = raw.strip()
        m = re.match(r"^(_Z\w+):", raw)
        if m:
            fn, queue, labels = m.group(1), [], {}
            i += 1
            continue
        m = re.match(r"^(\.LBB\w+):", raw)
        if m:
            labels[m.group(1)] = i
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
        if re.match(r"s_(buffer_)?load_", line):
            queue.append(None)
            i += 1
            continue
        if line.startswith("s_waitcnt"):
            m = re.search(r"lgkmcnt\((\d+)\)", line)
            if m:
                n = int(m.group(1))
                if n == 0:
                    queue = []
                elif all(e is not None for e in queue) and len(queue) > n:
                    queue = queue[len(queue) - n:]
            i += 1
            continue
        if line.startswith("s_endpgm"):
            if pending():
                report(i, "program end with reads in flight")
            i += 1
            continue
        if not line.startswith("s_"):
            if _regs(line) & pending():
                report(i, line)
        else:
            m = re.match(r"s_cbranch_\w+ (\.LBB\w+)", line)
            if m and m.group(1) in labels and (fn, i) not in rewalked:
                rewalked.add((fn, i))   # backward branch: once more round the loop with the present queue
                i = labels[m.group(1)]
                continue
        i += 1
    return issues
