"""Scans generated gfx950 assembly for MFMA register overlaps that the hardware does not allow.

An MFMA with a destination wider than four registers must not write registers it still reads as srcA /
srcB (the narrow forms, 16x16 results of four registers, read their operands before the first write and
may overlap).  The build runs this over every kernel's assembly and fails if such an instruction was
emitted.
"""
from __future__ import annotations

import re
import sys

_MFMA = re.compile(r"^\s*v_mfma_\w+\s+([av])\[(\d+):(\d+)\],\s*([av])\[(\d+):(\d+)\],\s*([av])\[(\d+):(\d+)\],\s*(\S+)")


def _overlap(a, b):
    return a[0] == b[0] and not (a[2] < b[1] or b[2] < a[1])


def find_overlaps(asm_text: str):
    bad = []
    for ln, line in enumerate(asm_text.splitlines(), 1):
        m = _MFMA.match(line)
        if not m:
            continue
        dst = (m.group(1), int(m.group(2)), int(m.group(3)))
        if dst[2] - dst[1] + 1 <= 4:
            continue
        src_a = (m.group(4), int(m.group(5)), int(m.group(6)))
        src_b = (m.group(7), int(m.group(8)), int(m.group(9)))
        if _overlap(dst, src_a) or _overlap(dst, src_b):
            bad.append((ln, line.strip()))
    return bad


_AREG = re.compile(r"\ba(\d+)\b|\ba\[(\d+):(\d+)\]")


def find_reserved_acc_uses(asm_text: str, kernel_pattern: str, reserved: int):
    """Kernels whose name matches kernel_pattern keep state in accumulation registers a0 .. a(reserved-1)
    that only their inline asm may touch (the compiler never sees those registers as values).  Returns the
    instructions OUTSIDE inline-asm blocks (the ;;#ASMSTART ... ;;#ASMEND regions of the emitted assembly)
    that name one of them."""
    bad = []
    in_kernel = in_asm = False
    for ln, line in enumerate(asm_text.splitlines(), 1):
        text = line.strip()
        if re.match(r"^[A-Za-z_.$][\w.$]*:", text):               # a label
            if not text.startswith(".L"):
                in_kernel = re.search(kernel_pattern, text) is not None
            continue
        if text.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if text.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not in_kernel or in_asm or not text or text.startswith((";", ".")):
            continue
        code = text.split(";")[0]
        for m in _AREG.finditer(code):
            lo = int(m.group(1)) if m.group(1) is not None else int(m.group(2))
            if lo < reserved:
                bad.append((ln, text))
                break
    return bad


if __name__ == "__main__":
    total = 0
    for path in sys.argv[1:]:
        for ln, text in find_overlaps(open(path).read()):
            print(f"{path}:{ln}: {text}")
            total += 1
    sys.exit(1 if total else 0)
