"""Builds the C-ABI library (csrc/*.hip -> libloco.so) for gfx950 with hipcc.

hipcc cross-compiles without a GPU.  The flags matter for correctness, not only for
speed: -ffp-contract=off keeps one rounding per written operation (the codes must be
reproducible bit for bit), division and square root stay correctly rounded, and the
target feature "packed-fp32-ops" is taken away from the device pass so that the compiler
selects no v_pk_add/mul/fma_f32 (tests/test_build_flags.py checks the device assembly).

The feature flag goes to both passes of hipcc; the HOST pass (x86-64) does not know an AMDGPU
feature and answers with one note per function set, "'-packed-fp32-ops' is not a recognized
feature for this target (ignoring feature)".  That note says nothing about the device pass,
where the flag does take effect, so build() drops exactly that line from what it prints.
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


HOST_FEATURE_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"


def without_host_feature_note(text: str) -> str:
    """hipcc's output minus the host pass's note about the device-only feature flag."""
    return "".join(line for line in text.splitlines(keepends=True) if line.strip() != HOST_FEATURE_NOTE)


def device_assembly(src: str | None = None) -> str:
    """The gfx950 assembly of the library's device code, built with the library's flags."""
    src = src or os.path.join(CSRC, "loco_api.hip")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [hipcc_path(), *flags, "-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", "-", src]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("hipcc -S failed (exit %d)" % res.returncode)
    return res.stdout


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
    if verbose:
        sys.stderr.write(without_host_feature_note(res.stderr))
    os.replace(tmp, out)
    return out


PROBE = os.path.join(HERE, "loco_traffic_probe")


def build_probe(out: str = PROBE) -> str:
    """The plain-C driver of the library for counter collection (csrc/loco_traffic_probe.c): gcc, C99,
    linked against libloco.so and the HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"),
           "-o", out, os.path.join(CSRC, "loco_traffic_probe.c"), "-L", HERE, "-lloco", "-L", os.path.join(rocm, "lib"),
           "-lamdhip64", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("gcc failed on the traffic probe (exit %d)" % res.returncode)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_probe())
