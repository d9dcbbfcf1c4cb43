"""Checks on the gfx950 assembly hipcc generates for the expert FFN kernel (text of `hipcc -S`, one kernel function at a time).

The streaming body of the kernel (csrc/ffn_bf16_tiled.hpp) requests its token operands with explicit load instructions
and waits for them with explicit `s_waitcnt vmcnt(N)` a few stages later.  Between the two the compiler believes the
registers already hold the data, so any instruction it places there that reads or writes them (a copy made by the register
allocator, a spill) would silently use stale values.  `in_flight_register_uses` finds such instructions.
"""
from __future__ import annotations

import re
from typing import Dict, List, Set, Tuple

TOKEN_LOAD = re.compile(r"^global_load_dwordx4 v\[(\d+):(\d+)\], v\[\d+:\d+\], off offset:(\d+)( sc1)?$")
EXPLICIT_WAIT = re.compile(r"^s_waitcnt vmcnt\((\d+)\)$")
VREG = re.compile(r"\bv(\d+)\b")
VRANGE = re.compile(r"\bv\[(\d+):(\d+)\]")


def kernel_functions(asm_text: str) -> Dict[str, List[str]]:
    """name -> instruction/marker lines of every `team::ffn_fused_kernel` instantiation in the file."""
    out = {}
    for m in re.finditer(r"^(_ZN4team16ffn_fused_kernel[^:\n]*):", asm_text, re.M):
        end = asm_text.find(".Lfunc_end", m.end())          # (a function may hold several s_endpgm: one per early exit)
        assert end > 0, m.group(1)
        out[m.group(1)] = [l.strip() for l in asm_text[m.end():end].split("\n")]
    return out


def registers(line: str) -> Set[int]:
    regs = {int(r) for r in VREG.findall(line)}
    for a, b in VRANGE.findall(line):
        regs.update(range(int(a), int(b) + 1))
    return regs


BODY_BEGIN, BODY_END = "; team_tiled_body_begin", "; team_tiled_body_end"


def streaming_bodies(lines: List[str]) -> List[List[str]]:
    """The instances of the streaming body inside a kernel function (the source marks where each begins and ends; they use
    different registers for their requests, so each is checked on its own); the whole function if it carries no marks."""
    bodies, cur = [], None
    for l in lines:
        if l == BODY_BEGIN:
            cur = []
        elif l == BODY_END and cur is not None:
            bodies.append(cur)
            cur = None
        elif cur is not None:
            cur.append(l)
    return bodies if bodies else [lines]


def in_flight_register_uses(lines: List[str]) -> Tuple[int, List[str]]:
    """Sum over the instances of the streaming body in a kernel function; see in_flight_register_uses_of_body."""
    total, found = 0, []
    for body in streaming_bodies(lines):
        n, v = in_flight_register_uses_of_body(body)
        total += n
        found += v
    return total, found


def in_flight_register_uses_of_body(lines: List[str]) -> Tuple[int, List[str]]:
    """(number of pipelined token-load groups found, violations).

    A group = the consecutive explicit token loads of one stage (both halves, both load flavours) with the last explicit
    counted wait (N > 0) in front of them; its window = from that wait to the loads.  From the first request in front of the
    loop to the last one inside it, a group's destination registers may be touched by compiler-generated instructions only inside its
    window: there the data has arrived (the matrix instructions read it, and once they have, the compiler may reuse the registers,
    e.g. for the address of the next request); anywhere else a request into them is still in flight."""
    in_asm = False
    events = []          # (index, kind, payload): 'load' (regs), 'wait' (N), 'ins' (text)
    for i, l in enumerate(lines):
        if "ASMSTART" in l:
            in_asm = True
            continue
        if "ASMEND" in l:
            in_asm = False
            continue
        if not l or l.startswith((";", ".", "//")) or l.endswith(":"):
            continue
        if in_asm:
            m = TOKEN_LOAD.match(l)
            if m:
                events.append((i, "load", set(range(int(m.group(1)), int(m.group(2)) + 1))))
                continue
            m = EXPLICIT_WAIT.match(l)
            if m:
                events.append((i, "wait", int(m.group(1))))
            continue
        events.append((i, "ins", l))
    # groups of loads: maximal runs of 'load' events not separated by a wait
    groups = []          # (first event pos, last event pos, regs, pos of last counted wait before the group or None)
    last_wait = None
    waits_since_group = 0
    k = 0
    while k < len(events):
        kind = events[k][1]
        if kind == "wait":
            if events[k][2] > 0:
                last_wait = k
                waits_since_group += 1
            k += 1
            continue
        if kind != "load":
            k += 1
            continue
        j, regs = k, set()
        while j < len(events) and events[j][1] != "wait" and (events[j][1] == "load" or j - k < 40):
            if events[j][1] == "load":
                regs |= events[j][2]
                last = j
            j += 1
        groups.append((k, last, regs, last_wait if waits_since_group else None))
        waits_since_group = 0
        k = last + 1
    pipelined = [g for g in groups if g[3] is not None]
    if not pipelined:
        return 0, []
    region = (groups[0][0], pipelined[-1][1])      # from the first request in front of the loop to the last one inside it
    violations = []
    for first, last, regs, wait_pos in pipelined:
        for pos in range(region[0], region[1] + 1):
            idx, kind, payload = events[pos]
            if kind != "ins":
                continue
            touched = registers(payload) & regs
            if not touched:
                continue
            inside = wait_pos < pos < first
            if not inside:
                violations.append(f"line {idx}: {payload}  (registers {sorted(touched)[:4]}.. of the loads at line {events[first][0]})")
    return len(pipelined), violations


VMEM = ("global_", "buffer_", "flat_", "scratch_")


def stale_scalar_base_uses(lines: List[str]) -> List[str]:
    """Explicit vector-memory instructions whose scalar base register was written by a vector instruction (v_readlane /
    v_readfirstlane: how the compiler brings a spilled or per-lane value back into a scalar register) fewer than five
    instructions earlier without idle cycles in between.  The hardware needs five wait states there; the compiler inserts them
    for its own memory instructions and cannot for one inside an `asm` statement."""
    found = []
    in_asm, first = False, True
    start = 0
    for i, l in enumerate(lines):
        if "ASMSTART" in l:
            in_asm, first, start = True, True, i
            continue
        if "ASMEND" in l:
            in_asm = False
            continue
        if not in_asm or not l or l.startswith(";"):
            continue
        if first and l.startswith("s_nop"):
            in_asm = False                      # the block starts with wait states
            continue
        first = False
        if not l.startswith(VMEM):
            continue
        regs = set(re.findall(r"\b(s\d+)\b", l))
        for a, b in re.findall(r"\bs\[(\d+):(\d+)\]", l):
            regs.update(f"s{r}" for r in range(int(a), int(b) + 1))
        if not regs:
            continue
        seen, j = 0, start - 1
        while j >= 0 and seen < 5:
            u = lines[j]
            if u and not u.startswith((";", ".")) and not u.endswith(":"):
                seen += 1
                m = re.match(r"(v_readlane_b32|v_readfirstlane_b32) (s\d+)", u)
                if m and m.group(2) in regs:
                    found.append(f"line {i}: {l}  after  {u}")
            j -= 1
    return found
