"""Compiles libbaklava.so in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libbaklava.so")

SOURCES = ["host_alloc.cpp", "api.hip", "decode_valu.hip", "decode_mfma.hip", "compact.hip", "profile.hip", "prefill.hip", "layer.hip", "probe.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 arithmetic is kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",  # MFMA accumulators stay in VGPRs (no AGPR copies)
    "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = True, out_path: str = LIB_PATH, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".hip") else ["-x", "hip", path])
    cmd += ["-o", out_path]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if verbose and out.strip():
        print(out)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out_path


if __name__ == "__main__":
    build_library()
    print("built", LIB_PATH)
