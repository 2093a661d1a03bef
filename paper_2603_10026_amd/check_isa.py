"""Build-time check of the hand-counted vector-memory waits.

Some kernels issue ``global_load_dwordx4`` into registers from inline assembly and wait for
the data with ``s_waitcnt vmcnt(N)`` statements written by hand, many instructions later.
The compiler sees each such statement as an ordinary definition of the destination
registers: it inserts no wait of its own, and nothing stops its register allocator from
copying or spilling a destination while the load is still in flight (a copy at a loop's
back edge, where the two unrolled halves of a pipeline chose different registers, is the
case that has been seen).  Such a copy reads the register's old contents and the kernel
computes garbage with no error.

This module compiles a source to gfx950 assembly (device code only) and walks each kernel
with a model of the two in-order counters: every vector-memory instruction joins one queue and
every LDS instruction another, ``s_waitcnt vmcnt(N)`` / ``lgkmcnt(N)`` retire all but the newest
N of their queue, and an instruction that names a register that a queued load will still write
is reported.  Scalar loads share the LDS counter but return out of order, so a partial
``lgkmcnt`` wait with a scalar load in flight is reported as well.  The walk follows the text from
top to bottom: a forward branch hands its state to its target, text behind an unconditional
branch is skipped until a label that has been handed a state, and where states meet the one
with the most operations in flight goes on.  Each backward branch is then taken once more from
its target with the queue it had at the branch, which covers the steady state of a
software-pipelined loop.

The same walk checks one hazard of inline-assembly dot instructions (``v_dot2c_f32_bf16`` and
its kin): their result may be read by an instruction of another kind only after three wait
states, which the compiler inserts behind dot instructions that it emits itself but not behind
one written in an ``asm`` statement.  An instruction counts as one wait state, ``s_nop N`` as
N + 1.  In a source that counts its own waits, a register spill inside a loop is reported as
well: the compiler waits for the reload with ``vmcnt(0)``, which drains every load the kernel
keeps in flight.  Likewise a scalar register written by a vector instruction (``v_readfirstlane_b32``,
``v_readlane_b32``) may be read by a vector-memory instruction only after five wait states;
the compiler sees to that for its own memory instructions, not for one inside an ``asm``
statement whose base address it has just moved to scalar registers.

``python -m paper_2603_10026_amd.check_isa file.hip [...]`` prints what it finds and exits
non-zero on a hazard.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

_VM_PREFIX = ("global_load", "global_store", "global_atomic", "buffer_load", "buffer_store",
              "buffer_atomic", "flat_load", "flat_store", "flat_atomic", "scratch_load",
              "scratch_store")
_REG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
_LABEL = re.compile(r"^([.\w$]+):")
_VMCNT = re.compile(r"vmcnt\((\d+)\)")
_LGKMCNT = re.compile(r"lgkmcnt\((\d+)\)")
_BRANCH = re.compile(r"^s_c?branch\w*\s+([.\w$]+)")


def _regs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1) is not None:
            out.add(int(m.group(1)))
        else:
            out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def _parse(asm_text):
    """Split an assembly file into kernels: name -> list of (kind, payload) entries."""
    kernels = {}
    cur = None
    for raw in asm_text.splitlines():
        line = raw.split(";")[0].rstrip()
        if not line.strip():
            continue
        m = _LABEL.match(line)
        if m:
            name = m.group(1)
            if not name.startswith(".L"):
                cur = kernels.setdefault(name, [])
            elif cur is not None:
                cur.append(("label", name))
            continue
        s = line.strip()
        if s.startswith(".") or cur is None:
            if s.startswith(".end_amdhsa_kernel") or s.startswith(".Lfunc_end"):
                cur = None
            continue
        if s.startswith("s_endpgm"):
            cur.append(("ins", s))
            continue
        cur.append(("ins", s))
    return {k: v for k, v in kernels.items() if any(e[1].startswith("s_endpgm") for e in v if e[0] == "ins")}


class Queues:
    """In-flight operations of the two counters that the kernels wait on by hand: vector
    memory (vmcnt) and LDS / scalar memory (lgkmcnt).  Entries are (registers, text, kind)."""

    def __init__(self, vm=None, lgkm=None, dots=None):
        self.vm = list(vm or [])
        self.lgkm = list(lgkm or [])
        self.dots = list(dots or [])   # [registers, text, wait states since] of recent dot instructions
        self.lane_reads = []           # [scalar registers, text, wait states since] of recent v_readlane's

    def copy(self):
        q = Queues(self.vm, self.lgkm, [list(d) for d in self.dots])
        q.lane_reads = [list(d) for d in self.lane_reads]
        return q


def _step(ins, q, where, report, counters=("vm", "lgkm")):
    """Apply one instruction to the queues of in-flight operations; hazards are reported for
    the named counters only."""
    mnem, _, ops = ins.partition(" ")
    _dot_hazard(mnem, ops, ins, q, where, report)
    if mnem == "s_waitcnt":
        m = _VMCNT.search(ops)
        if m:
            keep = int(m.group(1))
            del q.vm[: max(0, len(q.vm) - keep)]
        m = _LGKMCNT.search(ops)
        if m:
            keep = int(m.group(1))
            if keep == 0:
                q.lgkm.clear()
            elif any(kind == "smem" for _, _, kind in q.lgkm):
                # scalar loads return out of order: a partial wait proves nothing about LDS reads
                if "lgkm" in counters:
                    report.append(f"{where}: `{ins}` is a partial wait while a scalar load is in flight")
            else:
                del q.lgkm[: max(0, len(q.lgkm) - keep)]
        return
    named = _regs(ops)
    for dest, issued, _ in (q.vm if "vm" in counters else []) + (q.lgkm if "lgkm" in counters else []):
        hit = named & dest
        if hit:
            report.append(f"{where}: `{ins}` names v{min(hit)} while `{issued}` is in flight")
            break
    if mnem.startswith("ds_"):
        dest = set()
        if any(t in mnem for t in ("read", "load", "permute", "swizzle", "rtn")):
            dest = _regs(ops.split(",")[0])
        q.lgkm.append((dest, ins, "lds"))
        return
    if mnem.startswith(("s_load", "s_buffer_load")):
        q.lgkm.append((set(), ins, "smem"))
        return
    if mnem.startswith(_VM_PREFIX):
        dest = set()
        if "_load" in mnem and not re.search(r"\blds\b", ops) and "_lds_" not in mnem:
            dest = _regs(ops.split(",")[0])
        elif "atomic" in mnem and re.search(r"\b(sc0|glc)\b", ops):
            dest = _regs(ops.split(",")[0])
        q.vm.append((dest, ins, "vmem"))


_DOT_WAIT_STATES = 3
_LANE_READ_WAIT_STATES = 5
_SREG = re.compile(r"\bs(\d+)\b|\bs\[(\d+):(\d+)\]")


def _sregs(text):
    out = set()
    for m in _SREG.finditer(text):
        if m.group(1) is not None:
            out.add(int(m.group(1)))
        else:
            out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return out



def _dot_hazard(mnem, ops, ins, q, where, report):
    """Wait states between a dot instruction and a reader of another kind."""
    if q.dots and mnem.startswith("v_") and not mnem.startswith("v_dot"):
        named = _regs(ops)
        for dest, issued, age in q.dots:
            if age < _DOT_WAIT_STATES and named & dest:
                report.append(f"{where}: `{ins}` reads v{min(named & dest)} {age} wait states after `{issued}`")
                break
    passed = 1
    if mnem == "s_nop":
        try:
            passed = int(ops.strip(), 0) + 1
        except ValueError:
            passed = 1
    q.dots = [[d, t, a + passed] for d, t, a in q.dots if a + passed < _DOT_WAIT_STATES]
    if mnem.startswith("v_dot"):
        q.dots.append([_regs(ops.split(",")[0]), ins, 0])
    # scalar register written by a vector instruction, then read by a vector-memory instruction
    if q.lane_reads and mnem.startswith(_VM_PREFIX):
        named = _sregs(ops)
        for dest, issued, age in q.lane_reads:
            if age < _LANE_READ_WAIT_STATES and named & dest:
                report.append(f"{where}: `{ins}` reads s{min(named & dest)} {age} wait states after `{issued}`")
                break
    q.lane_reads = [[d, t, a + passed] for d, t, a in q.lane_reads if a + passed < _LANE_READ_WAIT_STATES]
    if mnem in ("v_readfirstlane_b32", "v_readlane_b32"):
        q.lane_reads.append([_sregs(ops.split(",")[0]), ins, 0])


def _longest(states):
    return max(states, key=lambda q: len(q.vm) + len(q.lgkm))


def _walk(name, entries, labels, start, end, state, counters, report, tag, back_edges=None):
    """Walk entries[start:end] in text order from `state`.  A forward branch hands a copy of the
    state to its target; after an unconditional branch the text is unreachable until a label
    that some branch has handed a state to.  Where several states meet, the one with the most
    operations in flight goes on.  Backward branches are recorded (with the state at the
    branch) in back_edges."""
    handed = {}
    for i in range(start, end):
        kind, p = entries[i]
        if kind == "label":
            incoming = handed.pop(i, [])
            if state is not None:
                incoming.append(state)
            state = _longest(incoming).copy() if incoming else None
            continue
        if state is None:
            continue
        m = _BRANCH.match(p)
        if m and m.group(1) in labels:
            target = labels[m.group(1)]
            if target > i:
                handed.setdefault(target, []).append(state.copy())
            elif back_edges is not None:
                back_edges.append((target, i, state.copy()))
            if p.startswith("s_branch"):
                state = None
            continue
        if p.startswith("s_endpgm"):
            state = None
            continue
        _step(p, state, f"{name} +{i}{tag}", report, counters)


def _successors(entries, labels, i):
    kind, p = entries[i]
    out = []
    if kind == "ins":
        if p.startswith("s_endpgm"):
            return out
        m = _BRANCH.match(p)
        if m and m.group(1) in labels:
            out.append(labels[m.group(1)])
            if p.startswith("s_branch"):
                return out
    if i + 1 < len(entries):
        out.append(i + 1)
    return out


def _reachable(entries, labels, start):
    """Entries that control can reach from `start`."""
    seen, todo = {start}, [start]
    while todo:
        for j in _successors(entries, labels, todo.pop()):
            if j not in seen:
                seen.add(j)
                todo.append(j)
    return seen


def _reaching(entries, labels, goal):
    """Entries from which control can reach `goal`."""
    preds = {}
    for i in range(len(entries)):
        for j in _successors(entries, labels, i):
            preds.setdefault(j, []).append(i)
    seen, todo = {goal}, [goal]
    while todo:
        for j in preds.get(todo.pop(), []):
            if j not in seen:
                seen.add(j)
                todo.append(j)
    return seen


def check_kernel(name, entries, counters=("vm", "lgkm")):
    """Return the list of hazards found in one kernel."""
    report = []
    labels = {p: i for i, (k, p) in enumerate(entries) if k == "label"}
    back_edges = []
    _walk(name, entries, labels, 0, len(entries), Queues(), counters, report, "", back_edges)
    for target, branch, q in back_edges:
        # from the label itself, so that the walk adopts the state handed to it
        _walk(name, entries, labels, target + 1, branch, q, counters, report, " (second trip)")
    if counters:
        # A register spilled inside a loop of a kernel that keeps its own loads in flight: the
        # compiler waits for its reload with vmcnt(0), which it believes is a wait for that one
        # load, and every request the kernel has in flight is waited for with it.
        for target, branch, _ in back_edges:
            # (a backward branch may also be the way back from a block laid out behind the
            # function's body: only what can reach the branch from its target is a loop)
            body = _reachable(entries, labels, target) & _reaching(entries, labels, branch)
            for i in sorted(body):
                kind, p = entries[i]
                if kind == "ins" and p.startswith("scratch_"):
                    report.append(f"{name} +{i}: `{p}` is a register spill inside a loop")
                    break
    seen, out = set(), []
    for r in report:
        key = r.split(": ", 1)[1]
        if key not in seen:
            seen.add(key)
            out.append(r)
    return out


def check_text(asm_text, counters=("vm", "lgkm")):
    hazards = []
    kernels = _parse(asm_text)
    for name, entries in kernels.items():
        hazards += check_kernel(name, entries, counters)
    return len(kernels), hazards


def check_source(path, hipcc, flags, counters=None):
    """Compile one HIP source to device assembly and check every kernel in it, for the counters
    that the source waits on by hand (see hand_counted) unless told otherwise."""
    if counters is None:
        counters = hand_counted(path)
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "dev.s")
        cmd = [hipcc, *flags, "--cuda-device-only", "-S", path, "-o", out]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc -S failed on {path}:\n{r.stdout}")
        with open(out) as f:
            return check_text(f.read(), counters)


def hand_counted(path):
    """The counters that a source waits on by hand: "vm" if it loads registers from global
    memory in inline assembly, "lgkm" if it reads LDS in inline assembly.  Loads that the
    compiler issues get the compiler's own waits; the model, which follows the text rather
    than the control flow, is not meant for them."""
    with open(path) as f:
        text = f.read()
    out = []
    if re.search(r'asm[^;]*global_load_dwordx\d %0', text):
        out.append("vm")
    if re.search(r'asm[^;]*"ds_read\w* %0', text):
        out.append("lgkm")
    return tuple(out)


if __name__ == "__main__":
    from . import build as _b
    bad = 0
    for src in sys.argv[1:]:
        n, hz = check_source(src, _b.hipcc(), _b.HIPCC_FLAGS)
        print(f"{src}: {n} kernels, {len(hz)} hazards")
        for h in hz:
            print("  " + h)
        bad += len(hz)
    sys.exit(1 if bad else 0)
