"""Static check of the compiled gemm_mid kernels: registers that asynchronous loads write.

gemm_mid loads X fragments and scales with `global_load_dword[x4]` instructions written as inline assembly and
waits for them itself (`s_waitcnt vmcnt(N)`, counted in issue order together with the LDS-direct loads).  The
compiler therefore does not know that such a register holds nothing until its load has landed: if it copied,
spilled, read or reused the register before the kernel's own wait, the kernel would compute with stale data or
have a register overwritten under it (an address register, say) when the load arrives.  The kernel marks the
point from which a destination may be used with an empty assembly statement that prints `; landed: <register>`
into the listing.  This module compiles the kernel source to assembly and checks, for every asynchronous load of
every gemm_mid kernel, that on each path to that marker (straight on, and once around the back edge of the K
loop) no instruction reads or writes the destination.

    python -m paper_2603_16590_amd.check_async_loads        # compiles, checks, prints one line per kernel
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

from .build import CSRC, FLAGS, HIPCC

_LOAD = re.compile(r"\tglobal_load_dword(?:x4)? v\[?(\d+)(?::(\d+))?\]?,")
_LANDED = re.compile(r"\t; landed: v\[?(\d+)(?::(\d+))?\]?")
_WRITE = re.compile(r"\t(?:v_\w+|ds_read\w*|global_load_dword(?:x4)?|scratch_load\w*|buffer_load\w*) v\[?(\d+)(?::(\d+))?\]?")
_NO_DST = re.compile(r"(global_store|ds_write|buffer_store|scratch_store|global_load_lds|global_atomic)")
_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def _range(a, b):
    a = int(a)
    return set(range(a, (int(b) if b else a) + 1))


def _writes(line):
    m = _WRITE.match(line)
    return _range(m.group(1), m.group(2)) if m else set()


def _reads(line):
    if not re.match(r"\t[a-z]", line):
        return set()
    parts = line.strip().split(None, 1)
    if len(parts) < 2:
        return set()
    has_dst = not _NO_DST.match(parts[0])
    out = set()
    for k, op in enumerate(parts[1].split(";")[0].split(",")):
        if k == 0 and has_dst:
            continue
        for m in _REG.finditer(op):
            out |= _range(m.group(1), m.group(2)) if m.group(1) else _range(m.group(3), None)
    return out


def check_listing(lines):
    """lines: the assembly of one kernel.  Returns (loads, violations) where violations is a list of strings."""
    labels = {}
    for i, ln in enumerate(lines):
        m = re.match(r"^(\.LBB\d+_\d+):", ln)
        if m:
            labels[m.group(1)] = i
    loops = []
    for i, ln in enumerate(lines):
        m = re.search(r"s_c?branch\w* (\.LBB\d+_\d+)", ln)
        if m and m.group(1) in labels and labels[m.group(1)] < i and any("v_mfma" in x for x in lines[labels[m.group(1)]:i]):
            loops.append((labels[m.group(1)], i))
    loads, bad = 0, []
    for i, ln in enumerate(lines):
        m = _LOAD.match(ln)
        if not m:
            continue
        loads += 1
        regs = _range(m.group(1), m.group(2))
        paths = [range(i + 1, len(lines))]
        for a, b in loops:
            if a <= i <= b:
                paths.append(list(range(i + 1, b + 1)) + list(range(a, len(lines))))
        for path in paths:
            marked = False
            for j in path:
                x = lines[j]
                lm = _LANDED.match(x)
                if lm and _range(lm.group(1), lm.group(2)) & regs:
                    marked = True
                    break
                if _reads(x) & regs or _writes(x) & regs:
                    bad.append("line %d: %s  -- touched at line %d: %s" % (i, ln.strip(), j, x.strip()))
                    marked = True
                    break
                if "s_endpgm" in x:
                    break
            if not marked:
                bad.append("line %d: %s  -- never marked as landed" % (i, ln.strip()))
    return loads, bad


def kernels_of(asm_text, name="gemm_mid"):
    """{mangled name: lines} of the kernels whose name contains `name`."""
    lines = asm_text.split("\n")
    out, start, cur = {}, None, None
    for i, ln in enumerate(lines):
        m = re.match(r"^(_Z\w+):", ln)
        if m:
            if cur is not None:
                out[cur] = lines[start:i]
            cur, start = (m.group(1), i) if name in m.group(1) else (None, None)
        elif cur is not None and ".amdhsa_kernel" in ln:
            out[cur] = lines[start:i]
            cur = None
    return out


def compile_listing(source="gemm_mxfp4.hip"):
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [HIPCC, *FLAGS, "--cuda-device-only", "-S", os.path.join(CSRC, source), "-o", out]
        p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if p.returncode != 0:
            raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), p.stdout))
        with open(out) as f:
            return f.read()


def main():
    ks = kernels_of(compile_listing())
    if not ks:
        raise SystemExit("no gemm_mid kernels in the listing")
    rc = 0
    for name, lines in ks.items():
        loads, bad = check_listing(lines)
        print("%s: %d asynchronous loads, %d violations" % (name, loads, len(bad)))
        for b in bad[:10]:
            print("   ", b)
        rc |= bool(bad) or loads == 0
    return rc


if __name__ == "__main__":
    sys.exit(main())
