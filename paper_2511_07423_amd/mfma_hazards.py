"""Static check of the compiler's output for the kernels that issue MFMAs from inline assembly.

The tall-tile GEMM kernels write their v_mfma_* instructions as inline assembly so that every
accumulator stays in one register for the whole K loop.  The price: the compiler does not know that an
accumulator was just written by the matrix core, so it neither inserts the wait states the hardware
needs before another instruction touches that register, nor avoids placing a register copy or a spill
right behind the MFMA.  The hardware does not interlock this case: the copy would silently read the
value from before the last accumulation.  The kernels therefore end every basic block with explicit
wait states; this module reads the generated assembly and verifies that the result is safe:

  after an MFMA that writes registers D, no instruction other than an MFMA that accumulates onto exactly D
  may name a register of D until `passes + 3` wait states have gone by (one per instruction, N + 1 for
  `s_nop N`), `passes` being 4 for the 16x16x32 and 8 for the 32x32x16 instructions;

  an MFMA may not read, as its first or second operand, a register that a vector-ALU instruction (the weight
  conversion, also inline assembly) wrote fewer than 2 wait states earlier.

Control flow is followed one level: at a branch, the instructions at the target are checked against the
MFMAs still settling at the branch.
"""
import re
import sys

_PASSES = {"v_mfma_f32_16x16x32_bf16": 4, "v_mfma_f32_32x32x16_bf16": 8, "v_mfma_f32_16x16x32_f16": 4}
_VALU_TO_MFMA_SRC = 2     # wait states between a vector-ALU write and an MFMA reading it as a source
_REG = re.compile(r"\b([av])(?:\[(\d+):(\d+)\]|(\d+))")


def _regs(text):
    """Set of (file, index) for every a/v register named in an operand string."""
    out = set()
    for m in _REG.finditer(text):
        if m.group(2) is not None:
            lo, hi = int(m.group(2)), int(m.group(3))
        else:
            lo = hi = int(m.group(4))
        out.update((m.group(1), i) for i in range(lo, hi + 1))
    return out


def _parse(lines):
    """-> (instructions [(mnemonic, operand text, source line no)], {label: index of the next instruction})."""
    ins, labels = [], {}
    for no, raw in enumerate(lines, 1):
        line = raw.split(";")[0].strip()
        if not line:
            continue
        if line.endswith(":"):
            labels[line[:-1]] = len(ins)
            continue
        if line.startswith("."):
            continue
        parts = line.split(None, 1)
        ins.append((parts[0], parts[1] if len(parts) > 1 else "", no))
    return ins, labels


def _states(mnemonic, operands):
    if mnemonic == "s_nop":
        return int(operands.strip(), 0) + 1
    return 1


def _touch(entry, pending, report, kernel):
    """Report `entry` if it names a register that an MFMA in `pending` [(dst regs, states left, line)] is still writing."""
    mn, ops, no = entry
    if mn == "s_nop":
        return
    if mn in _PASSES:
        fields = [f.strip() for f in ops.split(",")]
        dst, srcs, acc = _regs(fields[0]), _regs(fields[1]) | _regs(fields[2]), _regs(fields[3])
        hit = lambda regs: bool(regs & srcs) or (bool(regs & (dst | acc)) and not regs == dst == acc)
    else:
        used = _regs(ops)
        hit = lambda regs: bool(regs & used)
    for regs, left, at in pending:
        if hit(regs):
            report.append(f"{kernel}: line {no}: {mn} {ops} touches the result of the MFMA at line {at} "
                          f"with {left} wait states to go")


def _age(pending, entry):
    n = _states(entry[0], entry[1])
    return [(r, left - n, at) for r, left, at in pending if left - n > 0]


def check_kernel(name, lines):
    """Hazard messages for one kernel's assembly (list of lines; reported line numbers count from its label)."""
    ins, labels = _parse(lines)
    report, pending = [], []
    fresh = []                                    # (registers a vector-ALU instruction just wrote, states left, line)
    for entry in ins:
        mn, ops, no = entry
        _touch(entry, pending, report, name)
        if mn in _PASSES:
            fields = [f.strip() for f in ops.split(",")]
            srcs = _regs(fields[1]) | _regs(fields[2])
            for regs, left, at in fresh:
                if regs & srcs:
                    report.append(f"{name}: line {no}: {mn} {ops} reads a source written by the vector instruction "
                                  f"at line {at} with {left} wait states to go")
        fresh = _age(fresh, entry)
        if mn.startswith("v_") and mn not in _PASSES and not mn.startswith("v_cmp"):
            fresh.append((_regs(ops.split(",")[0]), _VALU_TO_MFMA_SRC, no))
        if mn.startswith(("s_cbranch", "s_branch")) and ops.strip() in labels and pending:
            ahead = list(pending)                 # the same MFMAs, seen from the branch target
            for target in ins[labels[ops.strip()]:]:
                if not ahead:
                    break
                _touch(target, ahead, report, name)
                ahead = _age(ahead, target)
        pending = _age(pending, entry)
        if mn in _PASSES:
            pending.append((_regs(ops.split(",")[0]), _PASSES[mn] + 3, no))
    return report


def check_file(path, name_filter="proj_kernel"):
    """Check every kernel of the assembly file whose symbol contains `name_filter` (a string or several).
    -> (number of kernels checked, number of inline MFMAs seen, hazard messages)"""
    with open(path) as f:
        lines = f.read().splitlines()
    filters = (name_filter,) if isinstance(name_filter, str) else tuple(name_filter)
    kernels, cur, name = [], None, None
    for no, line in enumerate(lines):
        m = re.match(r"^(_Z\w+):", line)
        if m and cur is None and any(f in m.group(1) for f in filters):
            name, cur = m.group(1), []
        elif cur is not None:
            if line.startswith(".Lfunc_end"):
                kernels.append((name, cur))
                cur = None
            else:
                cur.append(line)
    report, n_mfma = [], 0
    for name, body in kernels:
        n_mfma += sum(1 for l in body if l.strip().startswith("v_mfma"))
        report += check_kernel(name, body)
    return len(kernels), n_mfma, report


if __name__ == "__main__":
    n, n_mfma, rep = check_file(sys.argv[1], *(sys.argv[2:3]))
    print(f"{n} kernels, {n_mfma} MFMAs, {len(rep)} hazards")
    for r in rep[:40]:
        print(r)
    sys.exit(1 if rep else 0)
