"""Scan gfx950 assembly for vector instructions that read a register too soon after a matrix
instruction wrote it.

The matrix pipeline delivers its result some cycles after issue and the hardware does not
interlock a following vector-ALU read; the compiler pads with wait states.  It was seen to
leave a path uncovered (matrix instruction, two branches, a register copy of the accumulator:
3 to 4 wait states instead of 7), which gave wrong numbers in one build and not in the next.
This walks every control-flow path from each matrix instruction for NEED wait states and
reports vector-ALU reads of its destination inside that window.  `s_nop k` counts k + 1, any
other instruction 1; a register that is overwritten drops out of the dependence.
"""
import re

NEED = 7  # wait states between a 4-pass matrix instruction and a vector-ALU read of its result
_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def _regs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def _blocks(lines):
    blocks, order, cur = {"__entry": []}, ["__entry"], "__entry"
    for ln in lines:
        ln = ln.split(";")[0].rstrip()
        if not ln.strip():
            continue
        m = re.match(r"^(\.LBB[0-9_]+):", ln)
        if m:
            cur = m.group(1)
            blocks[cur] = []
            order.append(cur)
        elif not ln.lstrip().startswith("."):
            blocks[cur].append(ln.strip())
    return blocks, order


def scan(asm_text, name_filter="decode_kernel", need=NEED):
    """Returns [(kernel, block, matrix instruction, reader, wait states between them)]."""
    text = asm_text.split("\n")
    findings, kernels = [], 0
    i = 0
    while i < len(text):
        m = re.match(r"^(_Z\S+):", text[i])
        if not (m and name_filter in m.group(1)):
            i += 1
            continue
        j = i + 1
        while j < len(text) and "s_endpgm" not in text[j]:
            j += 1
        kernels += 1
        blocks, order = _blocks(text[i + 1 : j + 1])
        fallthrough = {}
        for bi, b in enumerate(order):
            ends_in_jump = bool(blocks[b]) and blocks[b][-1].startswith("s_branch")
            fallthrough[b] = order[bi + 1] if not ends_in_jump and bi + 1 < len(order) else None
        for b in order:
            for k, x in enumerate(blocks[b]):
                if not x.startswith("v_mfma"):
                    continue
                dst = frozenset(_regs(x.split()[1].rstrip(",")))
                seen, stack = set(), [(b, k + 1, 0, dst)]
                while stack:
                    bb, pos, ws, live = stack.pop()  # live: registers of the result not overwritten since
                    if ws >= need or not live or (bb, pos, live) in seen:
                        continue
                    seen.add((bb, pos, live))
                    ins, ended = blocks[bb], False
                    while pos < len(ins) and ws < need and live:
                        y = ins[pos]
                        op = y.split()[0]
                        nop = re.match(r"s_nop\s+(\d+)", y)
                        if nop:
                            ws += int(nop.group(1)) + 1
                            pos += 1
                            continue
                        parts = [p.strip() for p in y[len(op):].split(",")]
                        if op.startswith("v_") and not op.startswith("v_mfma"):
                            srcs = set()
                            for p in parts[1:]:
                                srcs |= _regs(p)
                            if srcs & live:
                                findings.append((m.group(1), bb, x, y, ws))
                                ended = True
                                break
                            if parts:
                                live = live - _regs(parts[0])
                        t = re.match(r"s_cbranch_\w+\s+(\S+)", y)
                        if t and t.group(1) in blocks:
                            stack.append((t.group(1), 0, ws + 1, live))
                        t = re.match(r"s_branch\s+(\S+)", y)
                        if t:
                            if t.group(1) in blocks:
                                stack.append((t.group(1), 0, ws + 1, live))
                            ended = True
                            break
                        ws += 1
                        pos += 1
                    if not ended and pos >= len(ins) and ws < need and live and fallthrough[bb]:
                        stack.append((fallthrough[bb], 0, ws, live))
        i = j
    return findings, kernels
