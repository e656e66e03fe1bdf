"""Builds libseer.so (the gfx950 HIP kernels plus the C ABI of include/seer.h) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libseer.so")
SOURCES = ["api.hip", "gate.hip", "decode_valu.hip", "decode_mfma.hip", "decode_merge.hip", "probe.hip", "frontend.hip", "train_fwd.hip"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def flags() -> list:
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, extra: list | None = None, out: str | None = None) -> str:
    """Compile every kernel for gfx950 and link the shared library (always recompiles)."""
    lib = out or LIB
    tmp = lib + f".tmp{os.getpid()}"
    cmd = [hipcc()] + flags() + (extra or []) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
