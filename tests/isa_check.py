"""Static check of the compiled kernels' ISA for the one hazard the hand-scheduled loads add.

The kernels request their streaming loads through inline asm and wait for them with explicit
``s_waitcnt vmcnt(N)``; the compiler therefore does not know which registers have a load in
flight.  It is free to copy, spill or reuse such a register, and any of those would read or
clobber data that has not landed yet.  This module compiles the kernels to assembly and scans
every kernel's control-flow graph: between a ``global_load`` issued from an inline-asm block and
the ``s_waitcnt vmcnt`` that retires it no other instruction, on any path, may name the load's
destination registers.  Loads, stores and atomics the compiler issues itself are counted (they share
the counter) but their registers are the compiler's business.
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

from paper_1912_12055_amd import build as _build

_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def _regs(text: str) -> set:
    out = set()
    for m in _REG.finditer(text):
        if m.group(1) is not None:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


_MAX_VARIANTS = 256


def _norm(pending: tuple) -> tuple:
    """Canonical form of an in-flight list: entries older than the oldest one that owns registers
    protect nothing, and the counter holds at most 63 requests (the machine stalls the issue of a
    64th until the oldest has retired)."""
    i = 0
    while i < len(pending) and not pending[i]:
        i += 1
    pending = pending[i:]
    return pending[-63:]


def _step(pending: tuple, lineno: int, t: str, op: str, bad: dict, in_asm: bool = True) -> tuple:
    return _norm(_step_raw(pending, lineno, t, op, bad, in_asm))


def _step_raw(pending: tuple, lineno: int, t: str, op: str, bad: dict, in_asm: bool) -> tuple:
    """Apply one instruction to one in-flight list (tuple of frozenset(dst regs), oldest first).

    Stores and atomics without return count in vmcnt on this target too and retire in issue order with
    the loads (the compiler's own wait insertion relies on it): they enter the list with no
    destination registers, so that a compiler-placed ``vmcnt(N)`` behind a run of stores retires the
    loads it is meant to."""
    if op == "s_waitcnt":
        m = re.search(r"vmcnt\((\d+)\)", t)
        if m:
            n = int(m.group(1))
            if n == 0:
                return ()
            if n < len(pending):
                return pending[len(pending) - n:]
        return pending
    if op.startswith("global_load") or op.startswith("buffer_load"):
        ops = t[len(op):].split(",")
        dst, src = _regs(ops[0]), _regs(",".join(ops[1:]))
        for rs in pending:
            if rs & (src | dst):
                bad.setdefault(lineno, f"{t}   [touches v{sorted(rs & (src | dst))}, destination of a load in flight]")
        # a load the compiler issued itself is tracked by the compiler (it may, for instance, load one
        # register from both arms of a divergent branch): it only takes its place in the count
        return pending + (frozenset(dst) if in_asm else frozenset(),)
    touched = _regs(t)
    for rs in pending:
        if rs & touched:
            bad.setdefault(lineno, f"{t}   [v{sorted(rs & touched)} is the destination of a load in flight]")
            break
    if op.startswith(("global_store", "buffer_store", "global_atomic", "buffer_atomic")):
        return pending + (frozenset(),)
    return pending


def check_kernel(lines, unmarked_is_asm: bool = True) -> list:
    """Violations [(line_no, text)] of one kernel.  ``unmarked_is_asm``: a listing without inline-asm markers is
    hand-written (every load in it is checked); compiled kernels pass False, so that a kernel that leaves all
    its loads to the compiler is not checked against the compiler's own, correct, bookkeeping.

    The kernel is split into basic blocks; the set of possible in-flight load lists is propagated
    along every control-flow edge to a fixed point (loads retire in order, so a list is trimmed to
    its N youngest entries by ``s_waitcnt vmcnt(N)``)."""
    insts = []  # (lineno, text, op, inside an inline-asm block)
    labels = {}
    in_asm = False
    marked = any("#ASMSTART" in raw for raw in lines) or not unmarked_is_asm
    for i, raw in enumerate(lines, 1):
        if "#ASMSTART" in raw:
            in_asm = True
        elif "#ASMEND" in raw:
            in_asm = False
        t = raw.split(";")[0].strip()
        if not t:
            continue
        if t.endswith(":"):
            labels[t[:-1]] = len(insts)
            continue
        if t.startswith("."):
            continue
        insts.append((i, t, t.split()[0], in_asm or not marked))
    if not insts:
        return []
    # basic block leaders
    leaders = {0} | set(labels.values())
    for k, (_, t, op, _a) in enumerate(insts):
        if op.startswith("s_cbranch") or op in ("s_branch", "s_endpgm", "s_setpc_b64"):
            leaders.add(k + 1)
    leaders = sorted(x for x in leaders if x < len(insts))
    block_of = {}
    for bi, start in enumerate(leaders):
        end = leaders[bi + 1] if bi + 1 < len(leaders) else len(insts)
        block_of[start] = (start, end)
    succs = {}
    for start, (s0, e0) in block_of.items():
        _, t, op, _a = insts[e0 - 1]
        out = []
        if op == "s_endpgm":
            pass
        elif op == "s_branch":
            out.append(labels[t.split()[1]])
        elif op.startswith("s_cbranch"):
            out.append(labels[t.split()[1]])
            if e0 < len(insts):
                out.append(e0)
        elif e0 < len(insts):
            out.append(e0)
        succs[start] = out
    bad = {}
    entry_states = {0: {()}}
    simulated = {}  # block -> entry states already pushed through it
    work = [0]
    while work:
        start = work.pop()
        s0, e0 = block_of[start]
        outs = set()
        fresh = entry_states[start] - simulated.setdefault(start, set())
        simulated[start] |= fresh
        for pend in fresh:
            cur = pend
            for k in range(s0, e0):
                ln, t, op, a = insts[k]
                cur = _step(cur, ln, t, op, bad, a)
            outs.add(cur)
        for nxt in succs[start]:
            have = entry_states.setdefault(nxt, set())
            new = outs - have
            if new:
                have |= new
                if len(have) > _MAX_VARIANTS:
                    raise RuntimeError("in-flight load analysis did not converge")
                work.append(nxt)
    return sorted(bad.items())


# the files whose kernels issue loads through inline asm (nna_train.hip leaves its loads to the compiler,
# which tracks them itself)
KERNEL_SOURCES = ("nna_kernels.hip", "nna_kernels_fold.hip", "nna_kernels_cqf.hip", "nna_kernels_f16.hip")


def compile_to_asm(extra_flags=()) -> str:
    """Device assembly of every kernel source file, concatenated."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in _build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    text = []
    with tempfile.TemporaryDirectory() as d:
        for src in KERNEL_SOURCES:
            out = os.path.join(d, src + ".s")
            cmd = [hipcc, *flags, *extra_flags, "-S", "--cuda-device-only", "-o", out, os.path.join(_build.CSRC, src)]
            subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
            text.append(open(out).read())
    return "\n".join(text)


def check_all(asm_text: str) -> dict:
    """{kernel symbol: [violations]} for every kernel in the assembly text."""
    src = asm_text.split("\n")
    starts = [(i, l.split(":")[0]) for i, l in enumerate(src) if re.match(r"^_Z\w+:", l)]
    res = {}
    for k, (i, name) in enumerate(starts):
        j = starts[k + 1][0] if k + 1 < len(starts) else len(src)
        body = src[i:j]
        end = next((x for x, l in enumerate(body) if l.startswith(".Lfunc_end")), len(body))
        res[name] = check_kernel(body[:end], unmarked_is_asm=False)
    return res


if __name__ == "__main__":
    total = 0
    for name, bad in check_all(compile_to_asm()).items():
        print(f"{name}: {len(bad)} violation(s)")
        for ln, msg in bad[:20]:
            print(f"   line {ln}: {msg}")
        total += len(bad)
    raise SystemExit(1 if total else 0)
