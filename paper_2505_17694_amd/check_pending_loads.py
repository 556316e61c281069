"""Checks the gfx950 assembly of kernels.hip for reads of registers that are still being loaded.

The dense path queues its query-row loads between asynchronous copies with inline assembly
(``ld16_pending``): the compiler does not know those registers are pending until the statement
that prints ``; query rows ready``, which the kernel places behind its own wait.  Nothing may touch
them in between, on any path, and nothing in the language guarantees that (a copy where two paths
join would be legal).  This script compiles the kernels to assembly, follows every path from each
pending load to the marker and fails if an instruction in between names one of the registers.

Run:  python -m paper_2505_17694_amd.check_pending_loads
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

from .build import CSRC, FLAGS, ROOT

MARKER = "query rows ready"
_LOAD = re.compile(r"\s*global_load_dwordx4 (v\[\d+:\d+\]), v\[\d+:\d+\], off\s*$")
_LABEL = re.compile(r"^(\.LBB\d+_\d+):")
_RANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_SINGLE = re.compile(r"\bv(\d+)\b")


def _regs(text: str) -> frozenset:
    out = set()
    for m in _RANGE.finditer(text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in _SINGLE.finditer(text):
        out.add(int(m.group(1)))
    return frozenset(out)


def assembly() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "kernels.s")
        cmd = [hipcc] + flags + ["-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                                 "-o", out, "-x", "hip", os.path.join(CSRC, "kernels.hip")]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc -S failed:\n" + res.stderr)
        with open(out) as f:
            return f.read()


def check(asm: str):
    """Returns (number of pending loads, number of markers, list of (line number, text) violations)."""
    lines = asm.splitlines()
    # nodes: instructions, pending loads and markers, in text order
    nodes = []          # (line index, kind, text)   kind: 'ins' | 'load' | 'mark'
    label_at = {}
    in_asm = False
    for i, raw in enumerate(lines):
        s = raw.strip()
        m = _LABEL.match(raw)
        if m:
            label_at[m.group(1)] = len(nodes)
            continue
        if s == ";;#ASMSTART":
            in_asm = True
            continue
        if s == ";;#ASMEND":
            in_asm = False
            continue
        if in_asm and MARKER in s:
            nodes.append((i, "mark", s))
            continue
        code = raw.split(";")[0].strip()
        if not code or code.startswith(".") or code.endswith(":"):
            continue
        if in_asm and _LOAD.match(raw):
            nodes.append((i, "load", code))
        else:
            nodes.append((i, "ins", code))
    succ = []
    for k, (_, _, code) in enumerate(nodes):
        op = code.split()[0]
        nxt = [k + 1] if k + 1 < len(nodes) else []
        if op == "s_endpgm":
            succ.append([])
        elif op == "s_branch":
            succ.append([label_at[code.split()[1]]])
        elif op.startswith("s_cbranch"):
            succ.append(nxt + [label_at[code.split()[1]]])
        else:
            succ.append(nxt)
    state = [frozenset()] * len(nodes)      # pending registers on entry
    work = [k for k, n in enumerate(nodes) if n[1] == "load"]
    loads, marks = len(work), sum(1 for n in nodes if n[1] == "mark")
    seen_out = {}
    while work:
        k = work.pop()
        _, kind, code = nodes[k]
        if kind == "load":
            out = state[k] | _regs(_LOAD.match(code).group(1))
        elif kind == "mark":
            out = frozenset()
        else:
            out = state[k]
        if seen_out.get(k) == out:
            continue
        seen_out[k] = out
        for t in succ[k]:
            merged = state[t] | out
            if merged != state[t] or t not in seen_out:
                state[t] = merged
                work.append(t)
    bad = []
    for k, (i, kind, code) in enumerate(nodes):
        if kind == "ins" and state[k] and (_regs(code) & state[k]):
            bad.append((i + 1, code))
    return loads, marks, bad


def main() -> int:
    loads, marks, bad = check(assembly())
    print(f"{loads} pending loads, {marks} markers, {len(bad)} instructions touch a pending register")
    for ln, code in bad[:40]:
        print(f"  line {ln}: {code}")
    return 1 if bad or not loads or not marks else 0


if __name__ == "__main__":
    sys.exit(main())
