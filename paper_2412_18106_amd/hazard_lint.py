"""Build-time check of the hand-issued instructions in the compiled kernels.

The attention kernel issues some MFMAs and LDS fragment reads as inline assembly
(see csrc/attn_kernels.hip for why).  The compiler schedules around them without
knowing what they are, so two things it normally guarantees have to be checked
on its output instead:

* the registers an inline-assembly MFMA writes are not read or written by any
  other kind of instruction (a register copy at a control-flow merge, a spill)
  before the wait states a vector-ALU access of an MFMA result needs have passed;
* the registers an inline-assembly ``ds_read`` writes are not touched before an
  ``s_waitcnt lgkmcnt`` has been issued;
* the registers an inline-assembly MFMA reads were not written by a vector-ALU
  instruction of the compiler's (a rematerialised constant, a copy) in the few
  wait states before it: the compiler pads that case for MFMAs it knows about.

* a scalar instruction in an inline-assembly statement that writes the SCC flag does not stand
  between a compare of the compiler's and the branch or select that reads it (the statement
  forgot to name "scc" among what it clobbers; met as a loop that never ended and then read
  out of bounds);

The check walks the assembly text of the device code straight down from each
such instruction to the end of its basic block.  It is conservative in one
direction only: everything it reports is a real hazard; a hazard that needs a
taken branch to happen is not seen.
"""
from __future__ import annotations

import re

MFMA_WAIT_STATES = 12        # what the compiler pads between a 32x32x16 bf16 MFMA and a vector-ALU use of its result

VALU_TO_MFMA_WAIT_STATES = 4  # vector-ALU write of a register -> MFMA reading it

# scalar instructions that write SCC / that read it
_SCC_WRITERS = re.compile(r"^s_(add|sub|addc|subb|addk|and|or|xor|nand|nor|xnor|andn2|orn2|lshl|lshr|ashr|bfe|min|max|abs|"
                          r"absdiff|not|cmp|cmpk|bcnt0|bcnt1|wqm|quadmask|lshl[1-4]_add)_")
_SCC_READERS = re.compile(r"^s_(cbranch_scc[01]|cselect_b32|cselect_b64|addc_u32|subb_u32|cmov_b32|cmov_b64)\b")

_reg = re.compile(r"\b([va])\[(\d+):(\d+)\]|\b([va])(\d+)\b")
_AGPR = 1000                 # accumulation registers are numbered from here


def _regs(text):
    out = set()
    for m in _reg.finditer(text):
        if m.group(1) is not None:
            base = _AGPR if m.group(1) == "a" else 0
            out.update(range(base + int(m.group(2)), base + int(m.group(3)) + 1))
        else:
            base = _AGPR if m.group(4) == "a" else 0
            out.add(base + int(m.group(5)))
    return out


def _operands(line):
    line = line.split(";")[0].strip()
    parts = line.split(None, 1)
    if len(parts) < 2:
        return parts[0] if parts else "", [], ""
    ops = [o.strip() for o in parts[1].split(",")]
    return parts[0], ops, parts[1]


def lint(asm_text):
    """Returns a list of (line number, message) for the hazards found in an AMDGPU assembly listing."""
    lines = asm_text.splitlines()
    in_asm = False
    problems = []
    for i, raw in enumerate(lines):
        s = raw.strip()
        if s.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if s.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not in_asm:
            continue
        op, ops, _rest = _operands(s)
        if _SCC_WRITERS.match(op):
            depth = 1
            for j in range(i + 1, len(lines)):
                t = lines[j].strip()
                if t.startswith(";;#ASMEND"):
                    depth -= 1
                    continue
                if t.startswith(";;#ASMSTART"):
                    depth += 1
                    continue
                if not t or t.startswith(";") or depth > 0:
                    continue
                if t.endswith(":") or t.startswith(".") or t.startswith("s_branch") or t.startswith("s_endpgm"):
                    break
                o2 = t.split()[0]
                if _SCC_READERS.match(o2):
                    problems.append((j + 1, f"'{t}' reads the SCC flag that the inline-assembly '{s}' at line {i + 1} "
                                            "wrote (the statement does not declare \"scc\" as clobbered)"))
                    break
                if _SCC_WRITERS.match(o2):
                    break
        if op.startswith("v_mfma"):
            src = _regs(",".join(ops[1:]))
            waited = 0
            asm_depth = 1            # walking up: inside this MFMA's own statement first
            for j in range(i - 1, -1, -1):
                t = lines[j].strip()
                if t.startswith(";;#ASMEND"):
                    asm_depth += 1
                    continue
                if t.startswith(";;#ASMSTART"):
                    asm_depth -= 1
                    continue
                if not t or t.startswith(";"):
                    continue
                if t.endswith(":") or t.startswith("."):
                    break
                o2, ops2, rest2 = _operands(t)
                if o2 == "s_nop":
                    waited += int(ops2[0]) + 1
                else:
                    # asm_depth is 0 on the compiler's own instructions, 1 inside an inline-assembly statement
                    if asm_depth == 0 and o2.startswith("v_") and not o2.startswith("v_mfma") and ops2 \
                            and _regs(ops2[0]) & src:
                        problems.append((i + 1, f"hand-issued MFMA reads a register that '{t}' (line {j + 1}) wrote "
                                                f"{waited} wait states earlier (needs {VALU_TO_MFMA_WAIT_STATES})"))
                        break
                    waited += 1
                if waited >= VALU_TO_MFMA_WAIT_STATES:
                    break
            dst = _regs(ops[0])
            waited = 0
            for j in range(i + 1, len(lines)):
                t = lines[j].strip()
                if not t or t.startswith(";"):
                    continue
                if t.endswith(":") or t.startswith(".") or t.startswith("s_cbranch") or t.startswith("s_branch") \
                        or t.startswith("s_endpgm") or t.startswith("s_barrier"):
                    break
                o2, ops2, rest2 = _operands(t)
                if o2 == "s_nop":
                    waited += int(ops2[0]) + 1
                elif o2.startswith("v_mfma"):
                    waited += 1       # the matrix pipe orders MFMAs among themselves
                else:
                    if _regs(rest2) & dst:
                        problems.append((j + 1, f"'{t}' touches the result of the hand-issued MFMA at line {i + 1} "
                                                f"after {waited} wait states (needs {MFMA_WAIT_STATES})"))
                        break
                    waited += 1
                if waited >= MFMA_WAIT_STATES:
                    break
        elif op.startswith("ds_read"):
            dst = _regs(ops[0])
            for j in range(i + 1, len(lines)):
                t = lines[j].strip()
                if not t or t.startswith(";"):
                    continue
                if t.endswith(":") or t.startswith(".") or t.startswith("s_cbranch") or t.startswith("s_branch") \
                        or t.startswith("s_endpgm"):
                    break
                o2, ops2, rest2 = _operands(t)
                if o2 == "s_waitcnt" and "lgkmcnt" in rest2:
                    break
                if o2 == "s_barrier":
                    continue
                if _regs(rest2) & dst:
                    problems.append((j + 1, f"'{t}' touches the destination of the hand-issued LDS read at line {i + 1} "
                                            "before any s_waitcnt lgkmcnt"))
                    break
    return problems
