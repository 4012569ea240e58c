"""Build-time check of the rotation kernels that load a row with inline-assembly `global_load_dwordx4`.

The compiler takes the destination registers of such a statement for defined where the statement stands; the data
arrives later, and every use in the source goes through an `s_waitcnt vmcnt(n)` statement tied to that register.
Nothing in the language stops the register allocator from copying or spilling such a register in between, so the
property is checked on the generated code: between each of these loads and the wait that releases it, no
instruction may name one of its destination registers.

    python check_asm_loads.py <file.s>      exit status 0 = holds for every kernel that has such loads
"""
import re
import sys


def regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        out.add(int(m.group(1)))
    return out


def check_kernel(name, lines):
    """lines: the kernel's instructions in order.  Returns (number of loads checked, list of violations)."""
    loads = []
    for i, l in enumerate(lines):
        m = re.match(r"\s*global_load_dwordx4 v\[(\d+):(\d+)\], v\d+, s\[", l)      # the form the source writes
        if m:
            loads.append((i, set(range(int(m.group(1)), int(m.group(2)) + 1))))
    bad = []
    n = len(loads)
    pos = loads[-1][0] if loads else 0               # the waits follow the last load, in the order n-1, n-2, .., 0
    for k, (i, dest) in enumerate(loads):
        release = None
        for j in range(pos + 1, len(lines)):
            m = re.match(r"\s*s_waitcnt vmcnt\((\d+)\)\s*$", lines[j].split(";")[0])
            if m and int(m.group(1)) == n - 1 - k:
                release = j
                break
        if release is None:
            bad.append("%s: load %d has no releasing wait" % (name, k))
            continue
        pos = release
        for j in range(i + 1, release):
            text = lines[j].split(";")[0]
            if text.strip() and regs(text) & dest and not re.match(r"\s*global_load_dwordx4", text):
                bad.append("%s: load %d: '%s' touches v%s before its wait" % (name, k, text.strip(), sorted(dest)))
                break
    return n, bad


def main(path):
    text = open(path).read()
    total, problems = 0, []
    for m in re.finditer(r"^(_Z\w+):.*?\n(.*?)^\.Lfunc_end", text, flags=re.S | re.M):
        name, body = m.group(1), m.group(2)
        if "fwht4096_wave_kernel" not in name or "global_load_lds_dwordx4" not in body:
            continue                                     # only the staged wave-per-row kernels load rows this way
        lines = [l for l in body.split("\n") if l.strip() and not l.strip().startswith((";", "."))]
        n, bad = check_kernel(name, lines)
        total += n
        problems += bad
    for p in problems:
        print("check_asm_loads:", p)
    print("check_asm_loads: %d inline-assembly row loads checked in %s, %d problems" % (total, path, len(problems)))
    return 1 if problems or total == 0 else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1]))
