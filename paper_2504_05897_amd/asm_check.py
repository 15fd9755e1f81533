"""Build-time check of the device assembly for registers reused while a hand-issued load is in flight.

The prefill kernels issue their weight loads from inline assembly and wait for them with explicit
s_waitcnt vmcnt(N).  The compiler does not know that such a load completes later: a destination register
whose value it considers dead may be handed out again at once, as the destination of the next load or as
scratch for an address computation, and the data that lands afterwards then corrupts that value (seen once:
the clobbered value was an address and the launch faulted).  The sources keep every such register alive up
to a wait; this scan is the net under that rule.

The scan is linear over each kernel's text, with the hardware's counter model: every vector-memory
instruction enters a queue, s_waitcnt vmcnt(N) retires all but the youngest N.  While a hand-issued load is
queued, any instruction that writes one of its destination registers, or that reads one (as an address, as
store data, or as the source of a vector ALU instruction, e.g. a copy into another register file), is
reported.  Reads by the matrix instructions are not checked: the sources tie those to the waits, and the
compiler places some of them out of line, which a linear scan cannot follow.

Two more findings come out of the same scan.  A vector-memory instruction that the compiler emitted itself
(outside an inline-assembly block) while a hand-issued one is still queued is reported: it would be one of the
"younger operations" that every hand-counted wait allows to stay in flight, and the wait would then cover one
operation less than the source counted.  find_wait_count_errors (below) recounts the waits of the main loops.

Control flow is followed only as far as this: a label that execution cannot fall into (the instruction before
it is an unconditional branch or ends the program) starts from the queue of the branches seen so far that jump
to it (the longest of them), or from an empty queue if none was seen -- the compiler lays the alternative code
paths of a kernel one after the other, and the text after a loop's closing branch is then another path's start,
not the loop's exit.
"""
from __future__ import annotations

import re
from typing import Iterable, List, Set, Tuple

_SPLIT = re.compile(r",\s*(?![^\[]*\])")


def _vregs(operand: str) -> Set[int]:
    operand = operand.split(" ")[0]
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", operand)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", operand)
    return {int(m.group(1))} if m else set()


def _waits_for_all(lines: List[Tuple[int, str]], label: str) -> bool:
    """Whether the text at a label waits for every vector-memory operation before it does anything else (restoring
    the execution mask and other waits aside): the shared tail of several code paths that ends their loads' time in flight."""
    at = None
    for i, (_, raw) in enumerate(lines):
        if raw.split(";")[0].strip() == label + ":":
            at = i
            break
    if at is None:
        return False
    for _, raw in lines[at + 1:]:
        text = raw.strip()
        if text.startswith(";;#ASM"):
            continue
        text = text.split(";")[0].strip()
        if not text:
            continue
        op, _, rest = text.partition(" ")
        if op in ("s_or_b64", "s_mov_b64") and rest.strip().startswith("exec"):
            continue
        if op == "s_waitcnt" and "vmcnt" not in rest:   # a wait for LDS or scalar loads
            continue
        return op == "s_waitcnt" and "vmcnt(0)" in rest
    return False


def _scan_kernel(name: str, lines: Iterable[Tuple[int, str]]) -> List[str]:
    lines = list(lines)
    # (destination registers of a hand-issued load or empty, line, issued from inline assembly)
    queue: List[Tuple[Set[int], int, bool]] = []
    found: List[str] = []
    in_asm = False
    jumps = {}            # label -> queue at each branch to it seen so far (by the branch's line)
    no_fall_through = False
    seen_labels = {}      # label -> lines of the hand-issued register loads that were queued when it was scanned
    # the closing branches of the main loops: the only backward branches a load may be in flight across (what
    # happens there is recounted by find_wait_count_errors)
    loops = _loops(lines)
    closing = {lines[b][0] for a, b in loops
               if not any((x, y) != (a, b) and a <= x and y <= b for x, y in loops) and _falls_through(lines[a:b + 1])}
    for no, raw in lines:
        text = raw.strip()
        if text.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if text.startswith(";;#ASMEND"):
            in_asm = False
            continue
        text = text.split(";")[0].strip()
        if text.endswith(":") and not text.startswith(".L") or not text:
            continue
        if text.endswith(":"):
            # What may be in flight here.  Without a path from above (or with one that has no hand-issued register load
            # in flight): the longest queue of the branches to the label seen so far.  Otherwise: the queue from above, and behind it (as if youngest: only a wait for everything retires
            # them) the hand-issued register loads that are in flight at such a branch and not on the path from above.
            arriving = list(jumps.get(text[:-1], {}).values())
            if no_fall_through or not any(hand and dest for dest, _, hand in queue):
                # (a path from above with no such load in flight adds nothing to what the branches bring)
                queue = list(max(arriving + ([] if no_fall_through else [queue]), key=len, default=[]))
                no_fall_through = False
            else:
                have = {line for _, line, _ in queue}
                for other in arriving:
                    for entry in other:
                        if entry[2] and entry[0] and entry[1] not in have:
                            queue.append(entry)
                            have.add(entry[1])
            seen_labels[text[:-1]] = {line for dest, line, hand in queue if hand and dest}
            continue
        if text.startswith("."):
            continue
        op, _, rest = text.partition(" ")
        if op in ("s_branch", "s_endpgm", "s_setpc_b64") or op.startswith("s_cbranch"):
            if op.startswith(("s_branch", "s_cbranch")):
                jumps.setdefault(rest.strip(), {})[no] = list(queue)
                if rest.strip() in seen_labels and no not in closing:
                    # A backward branch: if its target was scanned without a load that is in flight here, nothing
                    # has checked that text against it -- and where paths merge the compiler may copy or reuse
                    # registers.
                    loads = [line for dest, line, hand in queue if hand and dest and line not in seen_labels[rest.strip()]]
                    if loads and not _waits_for_all(lines, rest.strip()):
                        found.append("%s: line %d: %s goes back to %s while the hand-issued load of line %d may be in flight"
                                     % (name, no, op, rest.strip(), loads[0]))
            no_fall_through = not op.startswith("s_cbranch")
            continue
        no_fall_through = False
        ops = [o.strip() for o in _SPLIT.split(rest) if o.strip()] if rest else []
        if op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", rest)
            if m and int(m.group(1)) < len(queue):
                queue = queue[len(queue) - int(m.group(1)):] if int(m.group(1)) else []
            continue
        is_vmem = op.startswith(("global_", "flat_", "buffer_", "scratch_"))
        is_lds = op.startswith("ds_")
        is_load = is_vmem and "_load" in op and "_lds" not in op
        writes: Set[int] = set()
        addresses: Set[int] = set()
        has_dest = is_load or op.startswith("ds_read") or (
            op.startswith("v_") and not op.startswith(("v_cmp", "v_readfirstlane", "v_readlane")))
        if has_dest:
            writes = _vregs(ops[0]) if ops else set()
        if is_vmem or is_lds or (op.startswith("v_") and not op.startswith("v_mfma")):
            # sources: of memory instructions (addresses, store data) and of every vector ALU instruction but the
            # matrix ones (a copy to another register file is the typical case)
            for o in (ops[1:] if has_dest else ops):
                addresses |= _vregs(o)
        for dest, issued, _ in queue:
            if dest & writes:
                found.append("%s: line %d: %s writes v%s while the load of line %d may be in flight"
                             % (name, no, op, sorted(dest & writes), issued))
            if dest & addresses:
                found.append("%s: line %d: %s reads v%s while the load of line %d may be in flight"
                             % (name, no, op, sorted(dest & addresses), issued))
        if is_vmem:
            if not in_asm:
                older = [line for _, line, hand in queue if hand]
                if older:
                    found.append("%s: line %d: %s was emitted by the compiler while the hand-issued operation of line %d may be in "
                                 "flight: the hand-counted waits do not count it" % (name, no, op, older[0]))
            queue.append((writes if (is_load and in_asm) else set(), no, in_asm))
    return found


def find_inflight_hazards(asm_text: str) -> List[str]:
    """Scans every function of a device assembly listing; returns one message per finding."""
    found: List[str] = []
    name, lines = None, []
    for no, line in enumerate(asm_text.splitlines(), 1):
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name, lines = m.group(1), []
        elif line.startswith(".Lfunc_end"):
            if name:
                found += _scan_kernel(name, lines)
            name, lines = None, []
        elif name:
            lines.append((no, line))
    return found


# ---------------------------------------------------------------------------------------------------------------
# Recount of the hand-counted waits in the main loops.
#
# A main loop is the text from a label to the last branch back to it, if it holds no other such stretch and no
# unconditional branch before its end; branches out of it and forward branches inside it are taken as not taken,
# which gives the steady-state path (every K step present).  The body is
# walked several times with one queue of outstanding vector-memory operations, as the hardware keeps it, and from
# the second walk on:
#   * a matrix instruction may not read a register of a hand-issued load that a wait has not yet retired (the
#     wait in front of it allowed too many younger operations), and
#   * at a wait marked "opens an activation stage, ring of SA", every copy into LDS up to and including the stage
#     that is SA - 3 stages before the one last marked "activation stage issued" must have been retired: with a
#     ring of SA stages that is the stage the following barrier hands to the matrix instructions.
def _loops(lines: List[Tuple[int, str]]) -> List[Tuple[int, int]]:
    labels = {}
    out = {}
    for i, (_, raw) in enumerate(lines):
        text = raw.split(";")[0].strip()
        if text.endswith(":") and text.startswith(".L"):
            labels[text[:-1]] = i
            continue
        op, _, rest = text.partition(" ")
        if (op == "s_branch" or op.startswith("s_cbranch")) and rest.strip() in labels:
            out[labels[rest.strip()]] = i            # the last backward branch to a label closes its loop
    return sorted(out.items())


def _falls_through(body: List[Tuple[int, str]]) -> bool:
    """Whether execution that enters at the first line reaches the last one with every conditional branch not
    taken.  A label with a later branch back to it is not always a loop: the compiler also lays a block out in
    front of code that jumps back to it once (the block then leaves through an unconditional branch before the
    text reaches that jump)."""
    for _, raw in body[:-1]:
        op = raw.split(";")[0].strip().partition(" ")[0]
        if op in ("s_branch", "s_endpgm", "s_setpc_b64"):
            return False
    return True


def _scan_loop(name: str, body: List[Tuple[int, str]], walks: int = 5) -> List[str]:
    found: List[str] = []
    seen: Set[str] = set()
    queue: List[dict] = []
    stage = 0            # activation stages closed so far ("activation stage issued" marks seen)
    for walk in range(walks):
        in_asm = False
        for no, raw in body:
            text = raw.strip()
            if text.startswith(";;#ASMSTART"):
                in_asm = True
                continue
            if text.startswith(";;#ASMEND"):
                in_asm = False
                continue
            if in_asm and "hmoe: activation stage issued" in text:
                stage += 1
                continue
            code, _, comment = text.partition(";")
            code = code.strip()
            if not code or code.endswith(":") or code.startswith("."):
                continue
            op, _, rest = code.partition(" ")
            ops = [o.strip() for o in _SPLIT.split(rest) if o.strip()] if rest else []
            if op == "s_waitcnt":
                m = re.search(r"vmcnt\((\d+)\)", rest)
                if not m:
                    continue
                n = int(m.group(1))
                if n < len(queue):
                    queue = queue[len(queue) - n:] if n else []
                m = re.search(r"opens an activation stage, ring of (\d+)", comment)
                if m and walk >= 1:
                    must_have_landed = stage - 1 - (int(m.group(1)) - 3)
                    late = [q for q in queue if q["lds"] and q["stage"] <= must_have_landed]
                    msg = ("%s: line %d: s_waitcnt vmcnt(%d) opens an activation stage while %d of its copies into LDS (first: "
                           "line %d) may still be in flight" % (name, no, n, len(late), late[0]["line"] if late else 0))
                    if late and msg not in seen:
                        seen.add(msg)
                        found.append(msg)
                continue
            if op.startswith("v_mfma") and walk >= 1:
                reads: Set[int] = set()
                for o in ops[1:]:
                    reads |= _vregs(o)
                for q in queue:
                    if q["dest"] & reads:
                        msg = ("%s: line %d: %s reads v%s before a wait has retired the hand-issued load of line %d"
                               % (name, no, op, sorted(q["dest"] & reads), q["line"]))
                        if msg not in seen:
                            seen.add(msg)
                            found.append(msg)
                continue
            if op.startswith(("global_", "flat_", "buffer_", "scratch_")):
                is_lds = "_lds" in op
                is_load = "_load" in op and not is_lds
                queue.append({"dest": _vregs(ops[0]) if (is_load and in_asm and ops) else set(), "line": no,
                              "lds": is_lds and in_asm, "stage": stage})
    return found


def find_wait_count_errors(asm_text: str) -> List[str]:
    """Recounts the hand-counted waits of every main loop that issues loads from inline assembly; one message per
    finding."""
    found: List[str] = []
    name, lines = None, []
    for no, line in enumerate(asm_text.splitlines(), 1):
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name, lines = m.group(1), []
        elif line.startswith(".Lfunc_end"):
            if name:
                loops = _loops(lines)
                for first, last in loops:
                    # Only an innermost loop is one straight-line body that repeats; a loop around other loops (a
                    # block that works through several tiles) is walked through its inner loops.
                    if any((a, b) != (first, last) and first <= a and b <= last for a, b in loops):
                        continue
                    body = lines[first:last + 1]
                    if not _falls_through(body):
                        continue
                    text = "\n".join(raw for _, raw in body)
                    if "#ASMSTART" in text and "global_load" in text:
                        found += _scan_loop(name, body)
            name, lines = None, []
        elif name:
            lines.append((no, line))
    return found
