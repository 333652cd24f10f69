"""Static check of the compiled kernels' ISA for the one hazard the hand-scheduled loads add.

The kernels request their streaming loads through inline asm and wait for them with explicit
``s_waitcnt vmcnt(N)``; the compiler therefore does not know which registers have a load in
flight.  It is free to copy, spill or reuse such a register, and any of those would read or
clobber data that has not landed yet.  This module compiles the kernels to assembly and scans
every kernel linearly: between a ``global_load`` and the ``s_waitcnt vmcnt`` that retires it no
other instruction may name the load's destination registers.  (Control flow is ignored, which
makes the check conservative inside straight-line code and blind to loop back-edges; the
sources keep the in-flight registers in loop-carried variables with fixed roles for that
reason.)
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

from . import build as _build

_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def _regs(text: str) -> set:
    out = set()
    for m in _REG.finditer(text):
        if m.group(1) is not None:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def check_kernel(lines) -> list:
    """Violations [(line_no, text)] of one kernel's instruction list."""
    pending = []  # (line_no, destination registers), oldest first; stores hold an empty set
    bad = []
    for i, raw in enumerate(lines, 1):
        t = raw.split(";")[0].strip()
        if not t or t.endswith(":") or t.startswith("."):
            continue
        op = t.split()[0]
        if op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", t)
            if m:
                n = int(m.group(1))
                pending = pending[len(pending) - n:] if 0 < n < len(pending) else ([] if n == 0 else pending)
            continue
        if op.startswith("global_load") or op.startswith("buffer_load"):
            ops = t[len(op):].split(",")
            dst, src = _regs(ops[0]), _regs(",".join(ops[1:]))
            for ln, rs in pending:
                if rs & (src | dst):
                    bad.append((i, f"{t}   [touches registers of the load at line {ln}]"))
            pending.append((i, dst))
            continue
        if op.startswith("global_store") or op.startswith("buffer_store"):
            pending.append((i, set()))  # stores count in vmcnt as well
        touched = _regs(t)
        for ln, rs in pending:
            if rs & touched:
                bad.append((i, f"{t}   [v{sorted(rs & touched)} in flight since line {ln}]"))
                break
        if op == "s_endpgm":
            pending = []
    return bad


def compile_to_asm(extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in _build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "kernels.s")
        cmd = [hipcc, *flags, *extra_flags, "-S", "--cuda-device-only", "-o", out,
               os.path.join(_build.CSRC, "nna_kernels.hip")]
        subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        return open(out).read()


def check_all(asm_text: str) -> dict:
    """{kernel symbol: [violations]} for every kernel in the assembly text."""
    src = asm_text.split("\n")
    starts = [(i, l.split(":")[0]) for i, l in enumerate(src) if re.match(r"^_Z\w+:", l)]
    res = {}
    for k, (i, name) in enumerate(starts):
        j = starts[k + 1][0] if k + 1 < len(starts) else len(src)
        body = src[i:j]
        end = next((x for x, l in enumerate(body) if "s_endpgm" in l), len(body) - 1)
        res[name] = check_kernel(body[:end + 1])
    return res


if __name__ == "__main__":
    total = 0
    for name, bad in check_all(compile_to_asm()).items():
        print(f"{name}: {len(bad)} violation(s)")
        for ln, msg in bad[:20]:
            print(f"   line {ln}: {msg}")
        total += len(bad)
    raise SystemExit(1 if total else 0)
