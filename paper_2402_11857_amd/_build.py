"""Compiles the HIP library for gfx950 in-tree (paper_2402_11857_amd/libliec.so)."""
from __future__ import annotations

import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libliec.so")
SOURCES = [os.path.join(_HERE, "csrc", "liec_api.hip")]
HEADERS = [os.path.join(_HERE, "csrc", "liec_kernels.hpp"), os.path.join(_ROOT, "include", "liec.h"),
           os.path.join(_ROOT, "include", "liec_testing.h")] + \
          [os.path.join(_HERE, "csrc", "kernels", n)
           for n in ("common.hpp", "select.hpp", "sign.hpp", "step.hpp", "sync.hpp", "telemetry.hpp", "wire.hpp")]


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP library cannot be built")


def build_library(verbose: bool = False, defines=(), out: str = LIB_PATH) -> str:
    """Always recompiles.  -ffp-contract=off keeps every fp32 expression a single IEEE operation;
    packed fp32 instructions are disabled for the device pass.  `defines` (NAME=value strings) and `out`
    let a tuning run build a variant of the library beside the product's."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument"] + [f"-D{d}" for d in defines] + [
           "-I", os.path.join(_ROOT, "include"), "-I", os.path.join(_HERE, "csrc"),
           "-o", out] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose and res.stderr.strip():
        print(res.stderr)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
