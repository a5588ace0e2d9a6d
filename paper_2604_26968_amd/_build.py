"""Compiles csrc/*.hip into libkvm.so (gfx950).  Importable without the library."""
from __future__ import annotations

import glob
import os
import subprocess
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
# KVM_LIB names another build of the library for the binding to load (the host-sanitizer build of the
# CPU test suite); the default is the in-tree library.
LIB_PATH = os.environ.get("KVM_LIB") or os.path.join(_HERE, "libkvm.so")
SOURCES = ["kvm_util.hip", "kvm_score.hip", "kvm_state.hip", "kvm_select.hip", "kvm_pack.hip", "kvm_prefetch.hip", "kvm_dedup.hip"]


def build(verbose: bool = False, sanitize: bool = False, out: Optional[str] = None) -> str:
    """Run hipcc over every source, always (no staleness check); returns the library path.

    With ``sanitize`` the host side (argument validation, workspace carving, launch logic) is compiled
    with AddressSanitizer and UndefinedBehaviorSanitizer, the device code as usual; such a build must be
    given its own ``out`` path and needs the sanitizer runtime (:func:`asan_runtime`) preloaded."""
    out = out or os.path.join(_HERE, "libkvm.so")
    cmd = ["hipcc", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-pass-failed", "-Wno-inline-asm", "-I", _INCLUDE, "-I", _CSRC]
    if sanitize:
        assert os.path.abspath(out) != os.path.join(_HERE, "libkvm.so"), "a sanitizer build needs its own path"
        cmd += ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan"]
    else:
        cmd += ["-O3"]
    cmd += [os.path.join(_CSRC, s) for s in SOURCES]
    cmd += ["-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or r.returncode:
        noise = "not a recognized feature for this target"
        print("\n".join(l for l in (r.stdout + r.stderr).splitlines() if noise not in l))
    if r.returncode:
        raise RuntimeError("hipcc failed building %s" % out)
    return out


def asan_runtime() -> Optional[str]:
    """Path of the shared AddressSanitizer runtime of the compiler hipcc drives, or None."""
    for root in ("/opt/rocm/lib/llvm/lib/clang", "/opt/rocm/llvm/lib/clang"):
        hits = sorted(glob.glob(os.path.join(root, "*", "lib", "linux", "libclang_rt.asan-x86_64.so")))
        if hits:
            return hits[-1]
    return None
