"""Compiles csrc/*.hip into libkvm.so (gfx950).  Importable without the library."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
LIB_PATH = os.path.join(_HERE, "libkvm.so")
SOURCES = ["kvm_util.hip", "kvm_score.hip", "kvm_state.hip", "kvm_select.hip", "kvm_pack.hip", "kvm_prefetch.hip", "kvm_dedup.hip"]


def build(verbose: bool = False) -> str:
    """Run hipcc over every source, always (no staleness check); returns the library path."""
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-pass-failed", "-Wno-inline-asm", "-I", _INCLUDE, "-I", _CSRC]
    cmd += [os.path.join(_CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB_PATH]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or r.returncode:
        noise = "not a recognized feature for this target"
        print("\n".join(l for l in (r.stdout + r.stderr).splitlines() if noise not in l))
    if r.returncode:
        raise RuntimeError("hipcc failed building libkvm.so")
    return LIB_PATH
