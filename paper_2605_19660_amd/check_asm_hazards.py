"""Static checks of the compiled kernels for two hazards the compiler cannot see.

    python -m paper_2605_19660_amd.check_asm_hazards          (compiles to assembly, then scans)

A matrix instruction writes all registers of its destination when it retires, many clocks after
it was issued.  For its own instructions the compiler inserts the wait states the hardware asks
for before such a register is written again; the instructions inside an `asm` block it does not
look at.  If the register allocator places the output of an asm block on a destination register
of a matrix instruction that is still in flight -- which it may do when nobody reads that
register, e.g. the accumulator rows of absent heads -- the block's result is overwritten when the
matrix instruction retires.  This happened (run-to-run differences of the decode output in an
experimental build); the kernels now keep whole result tuples allocated until they have been
consumed (`keep_tuple`), and this scan checks the compiler's output for what is left:

    for every v_mfma: walk forward; an instruction that READS one of its destination registers
    (a dependent matrix instruction or a compiler-scheduled vector instruction, for which the
    compiler has inserted the wait states) proves that it has retired and ends the walk; an
    instruction inside ASMSTART/ASMEND that writes (or reads) one of them earlier, within
    `window` wait states, is reported.

The second check (every translation unit with DPP instructions in asm blocks): a DPP operand
must not be read in the two issue slots after a vector instruction wrote that register; the
compiler inserts the wait states for its own DPP instructions and for nothing inside an asm
block.  `scan_dpp` reports every DPP instruction between ASMSTART and ASMEND whose DPP source
register was written by one of the two vector instructions issued before it (an `s_nop n`
counts as n + 1 slots).
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ("oscar_decode_mfma.hip", "oscar_decode_mfma_zpmin.hip")
DPP_SOURCES = SOURCES + ("oscar_quantize.hip",)    # the encoder and the stand-alone rotations


def _regs(tok: str) -> set[int]:
    tok = tok.strip().rstrip(",")
    m = re.match(r"v\[(\d+):(\d+)\]$", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def _operands(text: str) -> list[set[int]]:
    parts = text.split(None, 1)
    if len(parts) < 2:
        return []
    return [_regs(o.split()[0]) if o.strip() else set() for o in parts[1].split(",")]


# Wait states after which a matrix instruction has certainly retired: the compiler's own tables ask
# for at most 19 between a matrix instruction's write and a vector write of the same register.
WINDOW = 24


def scan(asm_text: str, window: int = WINDOW) -> list[tuple]:
    lines = asm_text.split("\n")
    in_asm, flag = [False] * len(lines), False
    for i, l in enumerate(lines):
        if "#ASMSTART" in l:
            flag = True
        in_asm[i] = flag
        if "#ASMEND" in l:
            flag = False
    found, kernel = [], None
    for i, l in enumerate(lines):
        m = re.match(r"^(_Z\S+):", l)
        if m:
            kernel = m.group(1)
        t = l.strip()
        if not t.startswith("v_mfma"):
            continue
        pending = set(_operands(t)[0])          # destination registers not yet proven written
        waited = 0
        for j in range(i + 1, min(i + 200, len(lines))):
            tj = lines[j].strip()
            if not tj or tj[0] in ";." or tj.endswith(":"):
                if tj.endswith(":") and not tj.startswith(";"):
                    break                        # a label: control flow joins, stop here
                continue
            op = tj.split()[0]
            if op.startswith("s_cbranch") or op.startswith("s_branch") or op == "s_endpgm":
                break
            ops = _operands(tj)
            if op.startswith(("v_", "ds_", "buffer_", "global_")) and ops:
                is_store = op.startswith(("ds_write", "buffer_store", "global_store"))
                reads = set().union(*ops[1:]) if len(ops) > 1 and not is_store else set().union(*ops) if is_store else set()
                writes = set() if is_store else ops[0]
                if in_asm[j] and ((writes | reads) & pending):
                    found.append((kernel, i + 1, t, j + 1, tj, waited))   # (a read is no better)
                    pending -= writes | reads
                elif reads & pending:
                    break                        # a guarded read of any result register: the
                                                 # instruction has retired, all of them are written
                else:
                    pending -= writes            # rewritten by an instruction the compiler guards
            waited += int(tj.split()[1]) + 1 if op == "s_nop" else 1
            if waited > window or not pending:
                break
    return found


def scan_dpp(asm_text: str) -> list[tuple]:
    lines = asm_text.split("\n")
    found, flag, kernel = [], False, None
    recent: list[tuple[set[int], int]] = []      # (registers written, line) of the last vector instructions
    slots_since: list[int] = []                   # issue slots between each of them and now
    hist: list[tuple[set[int], int, int]] = []    # (written registers, line number, slots ago)
    for i, l in enumerate(lines):
        m = re.match(r"^(_Z\S+):", l)
        if m:
            kernel, hist = m.group(1), []
        if "#ASMSTART" in l:
            flag = True
        if "#ASMEND" in l:
            flag = False
        t = l.strip()
        if not t or t[0] in ";." or t.endswith(":"):
            if t.endswith(":") and not t.startswith(";"):
                hist = []                          # control flow joins: the compiler's own rules apply
            continue
        op = t.split()[0]
        step = int(t.split()[1]) + 1 if op == "s_nop" else 1
        if flag and "_dpp" in op:
            ops = _operands(t)
            src = ops[1] if len(ops) > 1 else set()      # the DPP operand is the first source
            for regs, ln, ago in hist:
                if ago < 2 and regs & src:
                    found.append((kernel, ln + 1, lines[ln].strip(), i + 1, t, ago))
        hist = [(r, ln, ago + step) for r, ln, ago in hist if ago + step < 4]
        if op.startswith("v_") and not op.startswith("v_cmp"):
            ops = _operands(t)
            if ops:
                hist.append((set(ops[0]), i, 0))
    return found


def compile_to_asm(source: str) -> str:
    from .build import COMMON, CSRC, SOURCES as BUILD_SOURCES
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = ["hipcc", *[c for c in COMMON if c != "-fPIC"], *BUILD_SOURCES.get(source, []),
               "--cuda-device-only", "-S", os.path.join(CSRC, source), "-o", out]
        subprocess.run(cmd, check=True, capture_output=True)
        return open(out).read()


def main() -> int:
    from concurrent.futures import ThreadPoolExecutor
    bad = 0
    with ThreadPoolExecutor(max_workers=3) as ex:
        texts = list(ex.map(compile_to_asm, DPP_SOURCES))
    for src, text in zip(DPP_SOURCES, texts):
        if src in SOURCES:
            n_mfma = text.count("\tv_mfma")
            found = scan(text)
            print("%s: %d matrix instructions, %d asm writes into a result still in flight" % (src, n_mfma, len(found)))
            for k, i, t, j, tj, w in found[:20]:
                print("  %s\n    line %d: %s\n    line %d (+%d wait states): %s" % (k, i, t, j, w, tj))
            bad += len(found)
        n_dpp = len(re.findall(r"#ASMSTART(?:(?!#ASMEND).)*?_dpp", text, re.S))
        found = scan_dpp(text)
        print("%s: %d asm blocks with DPP instructions, %d DPP reads inside two slots of the write" % (src, n_dpp, len(found)))
        for k, i, t, j, tj, ago in found[:20]:
            print("  %s\n    line %d: %s\n    line %d (%d slots later): %s" % (k, i, t, j, ago, tj))
        bad += len(found)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
