"""Check of the generated code of the kernels that manage their own load waits.

backward_coef_stream_kernel issues its vector loads and the waits for them as inline assembly.
Between such a load and its wait the destination registers are in flight, which the compiler
does not know: if it copies, moves or reuses them there, the kernel reads stale data and the
late load overwrites whatever the register was given to.  Nothing in the source can forbid
that, so the assembly is checked instead, at every build: on every path of the control flow
graph that starts after an inline-assembly load, the first instruction that names one of the
load's destination registers must be the wait that the source marks with "; landed <regs>" for
exactly those registers.  A path also ends at a wait for every outstanding load (vmcnt(0): the
kernel drains after its loop) or at the end of the program.

A second check reads the compiler's own resource report of the whole build (check_resources):
the kernels that carry a step hold their working set in registers by design (64 accumulators or
gy values per lane, a ring of table rows), a few registers below the limit of their occupancy,
and a change that pushes them over it does not fail, it spills to scratch memory inside the main
loop: such a build ran the cfg3 input gradient at 3.1 ms instead of 0.9 with every test green.
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

from . import build as hip_build

CHECKED_SOURCES = ("lmkan_backward.hip",)


def _regs(text: str) -> frozenset[int]:
    out: set[int] = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        out.add(int(m.group(1)))
    return frozenset(out)


def _functions(text: str):
    """(symbol, lines) of every kernel body in an assembly file."""
    for m in re.finditer(r"^(\w+):[^\n]*\n(.*?)^\s*s_endpgm", text, re.S | re.M):
        yield m.group(1), (m.group(2) + "\ts_endpgm").split("\n")


def check_function(symbol: str, lines: list[str]) -> tuple[int, list[str]]:
    """Number of inline-assembly loads found and the violations among them."""
    label_at = {}
    for i, l in enumerate(lines):
        m = re.match(r"^(\.?\w+):", l)
        if m:
            label_at[m.group(1)] = i
    code = [l.split(";")[0].strip() for l in lines]       # instruction text without comments
    marks = [l.split("; landed", 1)[1] if "; landed" in l else None for l in lines]

    def successors(i: int) -> list[int]:
        t = code[i]
        op = t.split()[0] if t else ""
        if op == "s_endpgm":
            return []
        if op in ("s_setpc_b64", "s_swappc_b64", "s_call_b64"):
            raise RuntimeError(f"{symbol}: indirect control flow at line {i}: {t}")
        if op == "s_branch":
            return [label_at[t.split()[1]]]
        if op.startswith("s_cbranch"):
            return [label_at[t.split()[1]], i + 1]
        return [i + 1] if i + 1 < len(lines) else []

    loads, in_asm = [], False
    for i, l in enumerate(lines):
        if "ASMSTART" in l:
            in_asm = True
        elif "ASMEND" in l:
            in_asm = False
        elif in_asm and re.match(r"(global|buffer)_load", code[i]):
            loads.append((i, _regs(code[i].split(None, 1)[1].split(",")[0])))

    bad = []
    for at, dst in loads:
        seen, todo = set(), successors(at)
        while todo:
            i = todo.pop()
            if i in seen:
                continue
            seen.add(i)
            if marks[i] is not None and _regs(marks[i]) == dst:
                continue                                  # the wait of this load: path done
            if re.match(r"s_waitcnt\b.*\bvmcnt\(0\)", code[i]):
                continue                                  # everything has landed
            if code[i] and not code[i].endswith(":") and not code[i].startswith(".") and _regs(code[i]) & dst:
                bad.append(f"{symbol}: load at line {at} ({lines[at].strip()}): "
                           f"line {i} touches its destination first: {lines[i].strip()}")
                continue
            todo.extend(successors(i))
    return len(loads), bad


def check_assembly(text: str) -> dict[str, int]:
    """Checks every kernel of an assembly file; returns {symbol: loads checked}, raises on a violation."""
    counts, bad = {}, []
    for symbol, lines in _functions(text):
        n, b = check_function(symbol, lines)
        if n:
            counts[symbol] = n
        bad += b
    if bad:
        raise RuntimeError("registers of in-flight loads are touched before their wait:\n  " + "\n  ".join(bad))
    return counts


def check(verbose: bool = False) -> dict[str, int]:
    """Compiles the checked sources to assembly with the flags of the library and checks them."""
    flags = [f for f in hip_build.FLAGS if f not in ("-shared", "-fPIC")]
    counts: dict[str, int] = {}
    with tempfile.TemporaryDirectory() as tmp:
        for name in CHECKED_SOURCES:
            out = os.path.join(tmp, name + ".s")
            cmd = [hip_build.HIPCC, *flags, "-S", "--cuda-device-only", "-o", out, os.path.join(hip_build.CSRC, name)]
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError("hipcc -S failed:\n" + res.stdout + res.stderr)
            with open(out) as f:
                got = check_assembly(f.read())
            if not got:
                raise RuntimeError(f"{name}: no inline-assembly loads found; the check no longer sees the kernel")
            counts.update(got)
    if verbose:
        for sym, n in counts.items():
            print(f"codegen check: {sym}: {n} loads, every one first touched by its wait", flush=True)
    return counts


if __name__ == "__main__":
    check(verbose=True)


# Kernels that must not touch scratch memory at all (substrings of the mangled names), and the
# most any kernel may use (bytes per lane: a few registers parked around a prologue are tolerated
# in the others, a spilled main loop is hundreds of bytes).
NO_SCRATCH = ("forward_slab_kernelIf", "forward_slab_f16_kernel", "backward_input_lane_kernel",
              "backward_input_slab_f16_kernel", "backward_coef_stream_kernel", "backward_fused_kernel",
              "hessian_reg_kernel", "head_kernel")
MAX_SCRATCH_BYTES = 64


def check_resources(report: str) -> dict[str, int]:
    """`report`: what hipcc prints with -Rpass-analysis=kernel-resource-usage.  Returns scratch bytes
    per lane of every kernel it lists; raises when a kernel breaks the limits above, or when the
    report lists no kernel at all."""
    scratch: dict[str, int] = {}
    name = None
    for line in report.split("\n"):
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"remark:\s+ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name is not None:
            scratch[name] = int(m.group(1))
    if not scratch:
        raise RuntimeError("resource check: the compiler's report names no kernel")
    bad = [f"{k}: {v} bytes of scratch per lane" for k, v in scratch.items()
           if v > MAX_SCRATCH_BYTES or (v > 0 and any(t in k for t in NO_SCRATCH))]
    if bad:
        raise RuntimeError("resource check: kernels spill registers to scratch memory\n  " + "\n  ".join(bad))
    return scratch
