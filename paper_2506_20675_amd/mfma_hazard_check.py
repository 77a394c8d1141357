"""Build-time check of the generated gfx950 assembly of this package's own kernels: how soon after a matrix-core
instruction (v_mfma_*) is its result read by anything that is not another v_mfma?

Why: the matrix cores deliver their result several issue slots after the instruction was issued, and an ordinary
instruction that reads the destination registers earlier sees the OLD accumulator.  The compiler pads such pairs with
s_nop, but its padding has been seen to fall short when the reader sits behind a TAKEN branch (register-allocator
copies of the accumulators, v_accvgpr_read_b32, at the head of a join block): the affected kernel then silently lost
the last low-order MFMA contribution of a wave's k range.  Nothing in the source can be pointed at, so the generated
code itself is checked after every build and the build fails when a reader is closer than MIN_SLOTS issue slots on
any path.

The scan works on `hipcc -S` output of our own source (labels, branches and instructions of each kernel), follows
both the fall-through and the branch target, counts one slot per instruction and n+1 per `s_nop n`, and stops a path
at MIN_SLOTS slots or when the destination registers are overwritten.
"""
from __future__ import annotations

import re
import sys

MIN_SLOTS = 8      # issue slots demanded between a v_mfma and the first non-MFMA reader of its destination: the distance
                   # the compiler itself keeps for v_mfma_f32_16x16x32_bf16 on gfx950 wherever its padding works

_REG = re.compile(r"\b([av])\[(\d+):(\d+)\]|\b([av])(\d+)\b")


def _regs(text: str) -> set:
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.update((m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1))
        else:
            out.add((m.group(4), int(m.group(5))))
    return out


def _parse_kernels(asm: str) -> dict:
    """-> {kernel name: list of (label or None, mnemonic, operand string)}"""
    kernels, cur, name = {}, None, None
    for raw in asm.splitlines():
        line = raw.split(";")[0].rstrip()
        if not line:
            continue
        m = re.match(r"^([A-Za-z_.$][\w.$]*):", line)
        if m and not line.startswith("\t"):
            lab = m.group(1)
            if not lab.startswith(".L"):            # a function symbol starts a new kernel body
                name, cur = lab, []
                kernels[name] = cur
            elif cur is not None:
                cur.append((lab, None, None))
            continue
        if cur is None or not line.startswith("\t") or line.strip().startswith("."):
            continue
        parts = line.strip().split(None, 1)
        cur.append((None, parts[0], parts[1] if len(parts) > 1 else ""))
        if parts[0] == "s_endpgm":
            cur = None
    return kernels


def _dst_src(mn: str, ops: str):
    """Destination and source register sets of one instruction (stores and compares have no register destination)."""
    fields = [f.strip() for f in ops.split(",")]
    no_dst = mn.startswith(("global_store", "scratch_store", "buffer_store", "flat_store", "ds_write", "ds_store",
                            "v_cmp", "s_", "v_cmpx"))
    if no_dst or not fields:
        return set(), _regs(ops)
    return _regs(fields[0]), _regs(",".join(fields[1:]))


def check(asm: str, min_slots: int = MIN_SLOTS) -> list:
    """-> list of (kernel, mfma line index, reader mnemonic + operands, slots) for every reader that is too close."""
    problems = []
    for kname, body in _parse_kernels(asm).items():
        labels = {lab: i for i, (lab, _, _) in enumerate(body) if lab}
        for i, (lab, mn, ops) in enumerate(body):
            if not mn or not mn.startswith("v_mfma"):
                continue
            dst, _ = _dst_src(mn, ops)
            # walk forward over all paths; state = (index, slots so far)
            seen, stack = {}, [(i + 1, 0)]
            while stack:
                j, slots = stack.pop()
                while j < len(body) and slots < min_slots:
                    if seen.get(j, min_slots + 1) <= slots:
                        break
                    seen[j] = slots
                    lab2, mn2, ops2 = body[j]
                    if not mn2:
                        j += 1
                        continue
                    d2, s2 = _dst_src(mn2, ops2)
                    if mn2.startswith("v_mfma"):
                        if d2 & dst:                       # accumulated into again (or overwritten): a new producer
                            break
                    else:
                        if (s2 | (d2 if mn2.startswith(("global_store", "scratch_store")) else set())) & dst:
                            problems.append((kname, i, f"{mn2} {ops2}", slots))
                            break
                        if d2 and d2 >= dst:
                            break
                    slots += (int(ops2.split()[0], 0) + 1) if mn2 == "s_nop" else 1
                    if mn2 == "s_endpgm":
                        break
                    if mn2 in ("s_branch",):
                        j = labels.get(ops2.strip(), len(body))
                        continue
                    if mn2.startswith("s_cbranch"):
                        t = labels.get(ops2.strip())
                        if t is not None:
                            stack.append((t, slots))
                    j += 1
    return problems


if __name__ == "__main__":
    text = open(sys.argv[1]).read()
    bad = check(text, int(sys.argv[2]) if len(sys.argv) > 2 else MIN_SLOTS)
    for k, i, what, slots in bad:
        print(f"{k}: result of v_mfma #{i} read after {slots} slots by: {what}")
    print(f"{len(bad)} reader(s) closer than the limit")
    sys.exit(1 if bad else 0)
