"""Build-time check of the gfx950 assembly that hipcc emits for this library's own kernels.

A matrix-core (MFMA) instruction delivers its result registers a fixed number of issue slots ("wait states") after it
issues, and a vector, LDS or memory instruction that touches those registers earlier reads what the registers held
before.  The hardware does not interlock this case; the compiler pads with s_nop.  Its padding has been seen to miss
a consumer that sits behind the TAKEN side of a uniform branch placed between the MFMA and the consumer (the
fall-through side was long enough, the taken side was one instruction): wrong gradients that depended on register
history, no fault, and gone with any change of instruction order.  The kernels are written so that every MFMA result
is consumed in the block that issues it; this scan fails the build if a future change (or compiler) breaks that.

For every MFMA the scan walks all paths forward (both sides of conditional branches) for the required number of wait
states and reports the first non-MFMA instruction that names one of its destination registers.
Required wait states before a VALU / LDS / memory access (CDNA3 ISA guide, "manually inserted wait states", with the
one extra state gfx950 needs for matrix instructions of four or more passes): passes + 2 for fp32 inputs,
passes + 3 (+ 1) otherwise; passes = cycles / 4.
"""
import re

# instruction shape -> wait states before a non-MFMA access of the result
NEED = {
    "f32_32x32x2_f32": 18,       # 16 passes, fp32 inputs
    "f32_16x16x4_f32": 10,       # 8 passes
    "f32_4x4x1_16b_f32": 4,      # 2 passes
    "f32_32x32x16_bf16": 12,     # 8 passes
    "f32_16x16x32_bf16": 8,      # 4 passes
}
DEFAULT_NEED = 20                # unknown shape: the longest rule

_LABEL = re.compile(r"^([.\w$]+):")
_RANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_SINGLE = re.compile(r"\bv(\d+)\b")


def _regs(text):
    out = set()
    for m in _RANGE.finditer(text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in _SINGLE.finditer(text):
        out.add(int(m.group(1)))
    return out


def _is_instruction(line):
    s = line.strip()
    return bool(s) and s[0] not in ";." and not _LABEL.match(s)


def scan(asm_text):
    """Returns a list of findings (strings); empty when every MFMA result is read late enough on every path."""
    lines = asm_text.split("\n")
    labels = {}
    for i, l in enumerate(lines):
        m = _LABEL.match(l)
        if m:
            labels[m.group(1)] = i
    findings = []
    func = "?"
    for i, l in enumerate(lines):
        m = re.match(r"^(_Z\w+):", l)
        if m:
            func = m.group(1)
        s = l.strip()
        if not s.startswith("v_mfma"):
            continue
        shape = s.split()[0][len("v_mfma_"):]
        need = NEED.get(shape, DEFAULT_NEED)
        dest = _regs(s.split(None, 1)[1].split(",")[0])
        stack = [(i + 1, 0)]
        seen = {}
        hit = None
        while stack and hit is None:
            j, w = stack.pop()
            while j < len(lines) and w < need:
                if not _is_instruction(lines[j]):
                    j += 1
                    continue
                if seen.get(j, need) <= w:
                    break
                seen[j] = w
                t = lines[j].strip().split(";")[0].strip()
                op = t.split()[0]
                if op == "s_endpgm":
                    break
                if op == "s_nop":
                    w += int(t.split()[1]) + 1
                elif op.startswith("v_mfma"):
                    # dependent matrix instructions are interlocked by the hardware; a new definition ends the walk
                    if _regs(t.split(None, 1)[1].split(",")[0]) & dest:
                        break
                    w += 1
                elif op == "s_branch":
                    j = labels[t.split()[1]]
                    w += 1
                    continue
                elif op.startswith("s_cbranch"):
                    stack.append((labels[t.split()[1]], w + 1))
                    w += 1
                else:
                    operands = t.split(None, 1)[1] if " " in t else ""
                    if op.startswith(("v_", "ds_", "global_", "buffer_", "flat_", "scratch_")) and _regs(operands) & dest:
                        hit = f"{func}: line {i + 1}: {s}\n    touched after {w} of {need} wait states at line {j + 1}: {t}"
                        break
                    w += 1
                j += 1
        if hit:
            findings.append(hit)
    return findings


def scan_file(path):
    with open(path) as f:
        return scan(f.read())
