"""Static check of the compiled kernels that issue transposing LDS reads from inline assembly.

The compiler does not know that such a read is still in flight after the statement, so nothing
but the kernel's own wait (an assembly statement that takes the same registers as operands) may
touch a destination register in between: a copy made earlier would hold stale data, and a
register handed to other code would be overwritten when the LDS data arrives.  This scans the
ISA for any instruction that names a pending destination register before a wait for all LDS
traffic, and for a transposing read whose address register is itself still pending."""
import re


def scan(asm_text: str):
    """Returns {function: [(line number, instruction), ...]} of hazards."""
    fn = None
    pending = set()
    issues = {}
    for i, raw in enumerate(asm_text.split("\n")):
        line = raw.strip()
        m = re.match(r"^(_Z\w+):", raw)
        if m:
            fn, pending = m.group(1), set()
            continue
        if not line or line[0] in ";.":
            continue
        m = re.match(r"ds_read_b64_tr_b16 v\[(\d+):(\d+)\], v(\d+)", line)
        if m:
            if int(m.group(3)) in pending:
                issues.setdefault(fn, []).append((i, line))
            pending.update(range(int(m.group(1)), int(m.group(2)) + 1))
            continue
        if line.startswith("s_waitcnt") and "lgkmcnt(0)" in line:
            pending.clear()
            continue
        if line.startswith("s_endpgm") and pending:
            issues.setdefault(fn, []).append((i, "program end with reads in flight"))
            continue
        if pending and not line.startswith("s_"):
            regs = set()
            for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", line):
                regs.update(range(int(a), int(b) + 1))
            for a in re.findall(r"\bv(\d+)\b", line):
                regs.add(int(a))
            if regs & pending:
                issues.setdefault(fn, []).append((i, line))
    return issues
