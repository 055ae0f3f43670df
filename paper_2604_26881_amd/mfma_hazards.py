"""Build-time check of the kernels' own assembly for two hazards the hardware does not interlock.

On CDNA an MFMA's result registers may not be read or overwritten by a non-MFMA instruction until
the matrix pipe has written them back: the ISA asks for a number of wait states (independent
instructions or s_nop) between the two that grows with the MFMA's passes (4 passes: 7, 8 passes:
11, 16 passes: 19).  The compiler pads with s_nop, but only along the straight-line order of the
code it emits: a conditional branch right behind a K loop's last MFMAs, whose target starts with
the epilogue's first reads of the accumulators, is not padded, and the epilogue then reads stale
accumulators (seen once in this library: one accumulator element per 32-column block wrong by
the last K slice's contribution).  This module follows every control-flow path backwards from each
instruction that touches an MFMA's result and fails the build if fewer wait states lie between.

A second, simpler check covers the other pair this library's code can get wrong: a load that writes LDS
(global_load_lds_*) takes its LDS address from m0 and needs one wait state after a scalar write of m0.
The compiler pads the pairs it emits itself, but the copies here are asm statements it does not look into.

It reads the device assembly hipcc writes for this library's own sources (-save-temps), nothing else.
"""
from __future__ import annotations

import re
from typing import Dict, Iterator, List, Optional, Tuple

# wait states between an MFMA and a non-MFMA instruction touching its result, by output shape of the bf16
# instructions this library uses (32x32x16: 8 passes, 16x16x32: 4 passes); anything else: the largest value
_WAIT_STATES = {"v_mfma_f32_32x32x16_bf16": 11, "v_mfma_f32_16x16x32_bf16": 7}
_DEFAULT_WAIT_STATES = 19
_REG = re.compile(r"\b([va])(?:(\d+)|\[(\d+):(\d+)\])")


def _registers(text: str) -> List[Tuple[str, int, int]]:
    """(file, first, last) of every vector register operand named in an operand string."""
    out = []
    for m in _REG.finditer(text):
        lo = int(m.group(2) if m.group(2) is not None else m.group(3))
        hi = int(m.group(2) if m.group(2) is not None else m.group(4))
        out.append((m.group(1), lo, hi))
    return out


def _kernels(path: str) -> Iterator[Tuple[str, List[str]]]:
    name: Optional[str] = None
    body: List[str] = []
    with open(path) as f:
        for line in f:
            m = re.match(r"^(\w+):\s*(;.*)?$", line)
            if m and name is None and not m.group(1).startswith("."):
                name, body = m.group(1), []
                continue
            if name is None:
                continue
            t = line.split(";")[0].strip()
            if not t:
                continue
            body.append(t)
            if t.startswith("s_endpgm"):
                yield name, body
                name = None


def hazards_in_kernel(body: List[str]) -> List[Tuple[str, str, int, int]]:
    """(mfma, touching instruction, wait states found, wait states needed) for every violation."""
    ins: List[str] = []
    labels: Dict[str, int] = {}
    for t in body:
        m = re.match(r"^(\.L\w+):$", t)
        if m:
            labels[m.group(1)] = len(ins)
            continue
        if t.startswith(".") or t.endswith(":"):
            continue
        ins.append(t)
    preds: Dict[int, List[int]] = {i: [] for i in range(len(ins))}
    for i, t in enumerate(ins):
        op = t.split()[0]
        if op.startswith("s_cbranch") or op == "s_branch":
            tgt = re.search(r"(\.L\w+)", t)
            if tgt and labels.get(tgt.group(1), len(ins)) < len(ins):
                preds[labels[tgt.group(1)]].append(i)
        if op != "s_branch" and not op.startswith("s_endpgm") and i + 1 < len(ins):
            preds[i + 1].append(i)

    def dest(i: int) -> Optional[Tuple[str, int, int]]:
        regs = _registers(ins[i].split(None, 1)[1].split(",")[0]) if " " in ins[i] else []
        return regs[0] if regs else None

    mfma_at = {i: dest(i) for i, t in enumerate(ins) if t.startswith("v_mfma")}
    found = []
    for i, t in enumerate(ins):
        op = t.split()[0]
        if op.startswith("v_mfma") or op.startswith("s_") or " " not in t:
            continue
        touched = _registers(t.split(None, 1)[1])
        if not touched:
            continue
        stack = [(p, 0) for p in preds[i]]
        best: Dict[int, int] = {}
        while stack:
            j, d = stack.pop()
            if d >= _DEFAULT_WAIT_STATES or best.get(j, 1 << 30) <= d:
                continue
            best[j] = d
            u = ins[j]
            uop = u.split()[0]
            if j in mfma_at and mfma_at[j] is not None:
                f, lo, hi = mfma_at[j]
                need = _WAIT_STATES.get(uop, _DEFAULT_WAIT_STATES)
                if d < need and any(tf == f and tlo <= hi and lo <= thi for tf, tlo, thi in touched):
                    found.append((u, t, d, need))
            w = int(u.split()[1], 0) + 1 if uop == "s_nop" else 1
            for p in preds[j]:
                stack.append((p, d + w))
    return found


def m0_hazards_in_kernel(body: List[str]) -> List[Tuple[str, str]]:
    """(m0 write, LDS-DMA load) pairs with no instruction between them.  A global/buffer load that writes LDS
    takes its LDS address from m0 and needs one wait state after a scalar write of m0; the pairs here come
    from this library's own asm statements, which the compiler does not pad."""
    ins = [t for t in body if not (t.startswith(".") or t.endswith(":"))]
    found = []
    for prev, cur in zip(ins, ins[1:]):
        op = cur.split()[0]
        if "_lds_" in op and op.startswith(("global_load", "buffer_load")) and prev.startswith("s_") \
                and re.match(r"^s_\w+\s+m0\b", prev):
            found.append((prev, cur))
    return found


def check_file(path: str) -> List[str]:
    """One line per kernel of the assembly file that has a violation."""
    out = []
    for name, body in _kernels(path):
        bad = hazards_in_kernel(body)
        if bad:
            u, t, d, need = min(bad, key=lambda b: b[2])
            out.append(f"{name}: {len(bad)} place(s) where an MFMA result is touched too early; the closest: "
                       f"`{t}` {d} wait states after `{u}` (needs {need})")
        m0 = m0_hazards_in_kernel(body)
        if m0:
            out.append(f"{name}: {len(m0)} LDS-writing load(s) directly behind the write of m0, e.g. `{m0[0][0]}` / `{m0[0][1]}`")
    return out
