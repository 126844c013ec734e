"""Build-time scan of the fast encoder's compiled assembly.

The fast encoder spells out its MFMA chains and some LDS reads as inline assembly, which the compiler schedules around
without knowing what the statements are: it does not insert the wait states an MFMA needs, and it may copy a register
that an LDS read has not filled yet.  The sources keep the required distances by construction; this scan checks the
generated code for the five ways the compiler could break them, so that a build that would compute wrong values
fails instead:
  1. an instruction other than the chain's next MFMA touches an MFMA's destination within 11 wait states of it
     (an 8-pass MFMA's result may be read after 11; an `s_nop N` counts N + 1);
  2. a register that an LDS read is still going to fill is touched before a wait on the LDS counter covers that read
     (the reads of a wavefront complete in order, so `lgkmcnt(N)` leaves the last N in flight);
  3. a vector instruction writes a source of an MFMA fewer than 2 wait states before it;
  4. a partial wait (`lgkmcnt(N)`, N > 0) is relied on for an LDS read while a scalar-memory load is in flight
     (those count on the same counter and return out of order, which makes the count meaningless);
  5. compiler-generated code reads SCC (`s_cselect`, `s_cbranch_scc*`, add/subtract with carry) when the last
     instruction that wrote it lies inside an inline-assembly statement: the statement changes SCC without saying so
     in its clobber list, and the compiler kept a condition in it across the statement.
"""
from __future__ import annotations

import re


def _regs(tok: str) -> set:
    out = set()
    for m in re.finditer(r"v\[(\d+):(\d+)\]", tok):
        out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"(?<![\w\[])v(\d+)\b", tok):
        out.add(int(m.group(1)))
    return out


_FLOW = ("s_cbranch", "s_branch", "s_swappc", "s_setpc", "s_endpgm", "s_barrier")
_ASM_BEGIN, _ASM_END = "#asm_begin", "#asm_end"      # markers of inline-assembly statements (kept by scan_file)
_SCC_WRITERS = ("s_cmp", "s_and", "s_or", "s_xor", "s_nand", "s_nor", "s_xnor", "s_add", "s_sub", "s_lshl", "s_lshr",
                "s_ashr", "s_bfe", "s_abs", "s_min", "s_max", "s_not", "s_wqm", "s_bcnt", "s_bitcmp", "s_quadmask")
_SCC_READERS = ("s_cselect", "s_cbranch_scc", "s_addc", "s_subb", "s_cmov")


def _scan_scc(lines: list) -> list:
    found, in_asm, written_in_asm = [], False, False
    for l in lines:
        if l == _ASM_BEGIN:
            in_asm = True
        elif l == _ASM_END:
            in_asm = False
        elif l.startswith(_SCC_READERS):
            if written_in_asm and not in_asm:
                found.append(f"SCC read after an inline-assembly statement wrote it: `{l}`")
                written_in_asm = False
            if l.startswith(("s_addc", "s_subb")):          # these write it as well
                written_in_asm = in_asm
        elif l.startswith(_SCC_WRITERS):
            written_in_asm = in_asm
        elif l.startswith(("s_swappc", "s_setpc")):
            written_in_asm = False                           # SCC does not survive a call
    return found


def scan_kernel(lines: list) -> list:
    """lines: the instructions of one kernel, in order (labels, comments and directives removed)."""
    found = _scan_scc(lines)
    lines = [l for l in lines if l not in (_ASM_BEGIN, _ASM_END)]
    inflight = []          # destinations of the LDS / scalar-memory operations not yet waited for, in issue order
    smem = False           # a scalar-memory operation is among them
    for i, l in enumerate(lines):
        pending = set().union(*inflight) if inflight else set()
        if l.startswith("v_mfma"):
            dst = _regs(l.split(",")[0])
            ws, j = 0, i + 1
            while j < len(lines) and ws < 11:
                n = lines[j]
                if n.startswith("s_nop"):
                    ws += int(n.split()[1]) + 1
                else:
                    if n.startswith("v_mfma"):
                        if _regs(n.split(",")[0]) == dst:
                            break                      # the chain goes on: the hardware handles this dependency
                    elif n.startswith(_FLOW):
                        break
                    elif _regs(n) & dst:
                        found.append(f"MFMA result touched after {ws} wait states: `{l}` then `{n}`")
                        break
                    ws += 1
                j += 1
            src = set()
            for tok in l.split(",")[1:]:
                src |= _regs(tok)
            ws, j = 0, i - 1
            while j >= 0 and ws < 2:
                n = lines[j]
                if n.startswith("s_nop"):
                    ws += int(n.split()[1]) + 1
                else:
                    if (n.startswith("v_") and not n.startswith(("v_mfma", "v_cmp")) and _regs(n.split(",")[0]) & src):
                        found.append(f"MFMA source written {ws} wait states before it: `{n}` then `{l}`")
                        break
                    ws += 1
                j -= 1
        if l.startswith("ds_read"):
            inflight.append(_regs(l.split(",")[0]))
        elif l.startswith(("ds_", "s_load", "s_memtime", "s_memrealtime", "s_buffer_load")):
            inflight.append(set())                     # counts on the same counter, fills no vector register
            smem = smem or l.startswith("s_")
        elif l.startswith("s_waitcnt") and "lgkmcnt(" in l:
            n = int(re.search(r"lgkmcnt\((\d+)\)", l).group(1))       # LDS operations complete in order
            if n and smem and pending:
                found.append(f"partial wait with a scalar-memory load in flight: `{l}`")
            inflight = inflight[len(inflight) - n:] if n else []
            smem = smem and n > 0
        elif l.startswith("s_swappc") and pending:
            found.append(f"call while LDS reads are in flight: `{l}`")
        elif pending and not l.startswith(_FLOW) and (_regs(l) & pending):
            found.append(f"register of an LDS read in flight touched: `{l}`")
    return found


def scan_file(path: str, kernel_filter: str) -> dict:
    """Scan every kernel of the assembly file whose symbol contains kernel_filter.  Returns {symbol: findings}."""
    out, name, cur = {}, None, []
    for raw in open(path):
        t = raw.strip()
        m = re.match(r"^(\w+):\s*(;.*)?$", t)
        if m and not t.startswith(".L") and raw[0] not in " \t":
            if name is not None:
                out[name] = scan_kernel(cur)
            name, cur = (m.group(1) if kernel_filter in m.group(1) else None), []
            continue
        if name is not None and t.startswith(";;#ASMSTART"):
            cur.append(_ASM_BEGIN)
        elif name is not None and t.startswith(";;#ASMEND"):
            cur.append(_ASM_END)
        if name is None or not t or t.startswith((";", ".", "//")) or t.endswith(":"):
            continue
        cur.append(t)
        if t.startswith("s_endpgm"):
            out[name] = scan_kernel(cur)
            name, cur = None, []
    return out
