"""Builds libdfa.so (the HIP kernels and the C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_PKG, "csrc")
INCLUDE = os.path.join(os.path.dirname(_PKG), "include")
LIB_PATH = os.path.join(_PKG, "libdfa.so")

SOURCES = ["dfa_api.hip", "dfa_fwd_bf16.hip", "dfa_fwd_f32.hip", "dfa_bwd.hip", "dfa_bwd_bf16.hip", "dfa_linear_bf16.hip", "dfa_dense.hip", "dfa_aux.hip", "dfa_probe.hip", "dfa_plan.cpp"]


def hipcc_command(out: str = LIB_PATH, extra=()):
    return ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            # keep the compiler from forming packed-fp32 instructions
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument",
            # the LDS-copy asm names m0 as clobbered; clang notes that it treats m0 as reserved anyway
            "-Wno-inline-asm",
            "-I", INCLUDE, *extra, "-o", out] + [os.path.join(CSRC, s) for s in SOURCES]


def build(verbose: bool = False) -> str:
    """Compiles every source into libdfa.so; raises on failure."""
    cmd = hipcc_command()
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libdfa.so")
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
