"""Static check of the assembly of kernels that issue LDS reads from inline asm and wait for them later.

Such a read names its destination registers as an asm output, so the compiler believes they hold the data as soon as
the asm statement ends; they do only after the `s_waitcnt lgkmcnt(n)` that covers the read.  The kernels are written
so that every use comes after that wait, but nothing stops the register allocator from placing a copy of such a
register between the read and the wait, which would silently copy stale data.  This check walks every kernel of an
assembly listing in program order, keeps the LDS operations that are still outstanding (they return in order, so a
wait for n leaves the newest n), and reports every instruction that reads or writes a register an outstanding read
is going to write (a later LDS read into the same registers excepted: it simply wins).  Branches are followed in layout order only, which is conservative for these kernels: their loops
begin with a wait for zero.  The build runs it on the compiler's output and fails on any finding."""
import re

_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def _regs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def kernels(asm_text):
    """(name, first line index, last line index) of every function in the listing."""
    lines = asm_text.split("\n")
    out = []
    i = 0
    while i < len(lines):
        m = re.match(r"^(_Z\w+):", lines[i])
        if m:
            j = i
            while j < len(lines) and not lines[j].strip().startswith("s_endpgm"):
                j += 1
            out.append((m.group(1), i, j))
            i = j
        i += 1
    return out


def violations(asm_text):
    """Findings as strings; empty when every register of an outstanding LDS read is left alone until its wait."""
    lines = asm_text.split("\n")
    found = []
    for name, first, last in kernels(asm_text):
        pending = []                      # (line index, destination registers), oldest first
        for i in range(first + 1, last):
            code = lines[i].split(";")[0].strip()
            if not code or code.startswith(".") or code.endswith(":"):
                continue
            op = code.split()[0]
            if op.startswith("s_waitcnt"):
                m = re.search(r"lgkmcnt\((\d+)\)", code)
                if m:
                    n = int(m.group(1))
                    pending = pending[len(pending) - n:] if n else []
                continue
            touched = _regs(code)
            if op.startswith("ds_read") or op.startswith("ds_load"):
                # another read into the same registers is harmless (LDS reads return in order: the later one wins);
                # only its address must not come from a register that is still to be delivered
                touched = _regs(code.split(",", 1)[1]) if "," in code else set()
            for at, dst in pending:
                if touched & dst:
                    found.append(f"{name}: line {i + 1} '{code}' touches v{sorted(touched & dst)} that the read at "
                                 f"line {at + 1} '{lines[at].strip()}' has yet to deliver")
            if op.startswith("ds_read") or op.startswith("ds_load"):
                pending.append((i, _regs(code.split(",")[0])))
            elif op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load"):
                pending.append((i, set()))          # counts towards lgkmcnt, delivers no vector register
    return found


if __name__ == "__main__":
    import sys
    bad = violations(open(sys.argv[1]).read())
    print("\n".join(bad) if bad else "no finding")
    sys.exit(1 if bad else 0)
