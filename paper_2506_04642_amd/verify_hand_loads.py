"""Build-time check of generated code (gfx950 assembly text) of the kernels that issue loads by hand.

csrc/decode_mfma.hip (global loads and LDS reads) and csrc/compressv.hip (LDS reads) issue some loads
by hand: the request and the hand-over of the destination registers to the compiler are separate
inline-assembly statements, with the wait between them.  In
between, the compiler believes that the destination already holds its value.  If it moves that value
(a copy into another register, a spill into the accumulation file or to scratch memory), it copies
stale contents, hands the register to something else, and the data then arrives on top of that --
wrong numbers at best, a wild address at worst.  Nothing in the language forbids such a move, so the
build reads what the compiler produced and refuses it unless, in every kernel,

  * every destination of a hand-issued `global_load_dwordx4 ... ; by hand` is handed over
    (`; by hand <registers>`) under the same name, and no instruction between the request and the
    hand-over names any of its registers;
  * no instruction between a hand-issued `ds_read_b128` (inside an inline-assembly block) and the
    next `s_waitcnt` with `lgkmcnt(0)` names a destination of such a read;
  * no scratch-memory instruction lies between a request and its hand-over.

The check follows the text in order, as the requests and hand-overs are written in straight-line code
(a wait may sit inside a branch, never a request or a hand-over); from reads at the end of a loop body
it follows the path that leaves the loop, not the back edge."""
import re
import sys

_REG = re.compile(r"\b([av])\[(\d+):(\d+)\]|\b([av])(\d+)\b")


def _regs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.update((m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1))
        else:
            out.add((m.group(4), int(m.group(5))))
    return out


def _code(line):
    c = line.split(";")[0].strip()
    if not c or c.startswith(".") or c.endswith(":"):
        return ""
    return c


def check_kernel(name, lines):
    """Problems found in one kernel's lines, as strings."""
    problems = []
    pending = {}   # line number of a global request -> its destination registers
    lds_pending = {}
    in_asm = False
    n_requests = n_lds = 0
    for no, line in lines:
        if "#ASMSTART" in line:
            in_asm = True
            continue
        if "#ASMEND" in line:
            in_asm = False
            continue
        if "global_load_dwordx4" in line and "by hand" in line:
            m = re.search(r"global_load_dwordx4\s+(\S+?),", line)
            dst = _regs(m.group(1))
            for at, regs in pending.items():
                if regs & dst:
                    problems.append("%s: line %d requests into registers still awaited from line %d" % (name, no, at))
            pending[no] = dst
            n_requests += 1
            continue
        if "; by hand" in line and "global_load" not in line:
            m = re.search(r"; by hand\s+(\S+)", line)
            got = _regs(m.group(1)) if m else set()
            hit = [at for at, regs in pending.items() if regs == got]
            if not hit:
                problems.append("%s: line %d hands over %s, which no request names" % (name, no, m.group(1) if m else "?"))
            for at in hit:
                del pending[at]
            continue
        code = _code(line)
        if not code:
            continue
        if in_asm and code.startswith("ds_read_b128"):
            m = re.match(r"ds_read_b128\s+(\S+?),", code)
            lds_pending[no] = _regs(m.group(1))
            n_lds += 1
            continue
        if code.startswith("s_waitcnt") and "lgkmcnt(0)" in code:
            lds_pending.clear()  # (whoever issued it: nothing read from LDS is still on its way)
            continue
        named = _regs(code)
        if pending:
            if code.startswith("scratch_"):
                problems.append("%s: line %d: scratch access while hand-issued loads are awaited" % (name, no))
            for at, regs in pending.items():
                if regs & named:
                    problems.append("%s: line %d `%s` names a register awaited from line %d" % (name, no, code, at))
        for at, regs in lds_pending.items():
            if regs & named:
                problems.append("%s: line %d `%s` names a register of the LDS read at line %d" % (name, no, code, at))
        if code.startswith("s_endpgm") and (pending or lds_pending):
            problems.append("%s: requests never handed over: lines %s" % (name, sorted(pending) + sorted(lds_pending)))
    return problems, n_requests, n_lds


def check_text(text, kernel="decode_split_mfma_kernel"):
    """(problems, kernels checked, hand-issued global requests, hand-issued LDS reads) of an assembly file;
    the kernels are the functions whose mangled name contains `kernel`."""
    lines = text.split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"_Z\S*" + re.escape(kernel) + r"\S*:\s*", l)]
    problems, kernels, total, total_lds = [], 0, 0, 0
    for k, a in enumerate(starts):
        b = len(lines)
        for j in range(a + 1, len(lines)):
            if lines[j].startswith(".Lfunc_end"):
                b = j
                break
        name = lines[a].split(":")[0]
        p, n, nl = check_kernel(name, [(i + 1, lines[i]) for i in range(a, b)])
        problems += p
        kernels += 1
        total += n
        total_lds += nl
    return problems, kernels, total, total_lds


def verify(path, kernel="decode_split_mfma_kernel", global_loads=True):
    """Raises RuntimeError if the assembly file at `path` breaks a rule above.  global_loads: the kernels
    are expected to hold hand-issued global loads (LDS reads are expected always)."""
    with open(path) as f:
        problems, kernels, total, total_lds = check_text(f.read(), kernel)
    if kernels == 0:
        raise RuntimeError("%s: no %s found: nothing was checked" % (path, kernel))
    if (global_loads and total == 0) or total_lds == 0:
        raise RuntimeError("%s: no hand-issued loads found in %d kernels: the check no longer sees them" % (path, kernels))
    if problems:
        raise RuntimeError("hand-issued loads: %d problem(s) in %s\n%s" % (len(problems), path, "\n".join(problems[:20])))
    return kernels, total, total_lds


if __name__ == "__main__":
    k, n, nl = verify(sys.argv[1], *(sys.argv[2:3] or ["decode_split_mfma_kernel"]), global_loads=len(sys.argv) < 3)
    print("%d kernels, %d hand-issued global loads, %d hand-issued LDS reads: registers untouched until handed over" % (k, n, nl))
