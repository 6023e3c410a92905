"""Builds libctc_mi355x.so for gfx950 with hipcc, in-tree next to this file.

    python -m paper_1512_02595_amd.build

hipcc cross-compiles without a GPU.  Packed-fp32 code generation is switched off
for all device code.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libctc_mi355x.so")
SOURCES = ["ctc_kernels.hip", "ctc_api.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def command(out: str = LIB) -> list[str]:
    return [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            # no NaN ever enters the arithmetic (log 0 is a finite sentinel): lets max/min
            # skip the quieting of their operands
            "-fno-honor-nans",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-x", "hip",
            "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
            *os.environ.get("CTC_EXTRA_HIPCC_FLAGS", "").split(),
            "-I", os.path.join(ROOT, "include"), "-I", CSRC,
            *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]


def build(verbose: bool = False) -> str:
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = command(tmp)
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building libctc_mi355x.so")
    if verbose and res.stderr.strip():
        sys.stderr.write(res.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
