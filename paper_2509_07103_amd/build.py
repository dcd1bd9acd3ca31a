"""Build the HIP library (liblmkan.so) for gfx950, in-tree, next to this file."""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblmkan.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed float32 VALU instructions are switched off: some of their forms have given
# silently wrong results on the target machines.  MFMA accumulators are kept in ordinary
# vector registers (gfx950 allows it): the coefficient-gradient kernel reads them with
# vector instructions at the end of every cell, and copies out of the accumulation
# registers would cost as much as the combine itself.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-munsafe-fp-atomics", "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    """Compiles the library; the compiler's resource report of the same run goes through
    check_codegen.check_resources, so a build whose hot kernels spill registers raises."""
    cmd = [HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", *(extra or []), "-o", LIB, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building liblmkan.so")
    # (what is left of stderr without the report and the source lines it quotes: warnings)
    other = "\n".join(line for line in res.stderr.split("\n")
                      if "kernel-resource-usage" not in line and not re.match(r"\s*\d*\s*\|", line))
    if verbose and other.strip():
        sys.stderr.write(other)
    from . import check_codegen
    scratch = check_codegen.check_resources(res.stderr)
    if verbose:
        print(f"resource check: {len(scratch)} kernels, {sum(1 for v in scratch.values() if v)} with scratch "
              f"(at most {max(scratch.values())} bytes per lane)", flush=True)
    return LIB


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(ROOT, "include", "lmkan.h")]
    return all(os.path.getmtime(d) <= t for d in deps)


if __name__ == "__main__":
    print(build(verbose=True))
    sys.path.insert(0, ROOT)
    from paper_2509_07103_amd import check_codegen
    check_codegen.check(verbose=True)
