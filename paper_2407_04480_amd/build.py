"""Builds the C-ABI library (csrc/*.hip -> libloco.so) for gfx950 with hipcc.

hipcc cross-compiles without a GPU.  The flags matter for correctness, not only for
speed: -ffp-contract=off keeps one rounding per written operation (the codes must be
reproducible bit for bit), division stays correctly rounded, and packed-fp32
instruction selection is switched off.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libloco.so")

# Extra -D definitions (none by default; the launch shapes live in csrc/loco_api.hip).
TUNING: dict = {}

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-ffp-contract=off",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall",
    "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the library cannot be built")


def build(out: str = LIB, tuning: dict | None = None, verbose: bool = False) -> str:
    """Compile every HIP source into one shared library; always recompiles."""
    defs = dict(TUNING)
    defs.update(tuning or {})
    srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc_path(), *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[f"-D{k}={v}" for k, v in defs.items()], "-o", tmp, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed (exit %d)" % res.returncode)
    if verbose and res.stderr.strip():
        sys.stderr.write(res.stderr)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
