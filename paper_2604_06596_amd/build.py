"""Compile the HIP library for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_SRC = os.path.join(_HERE, "csrc", "dynlp.hip")
_SO = os.path.join(_HERE, "libdynlp.so")


def library_path() -> str:
    return _SO


def build(verbose: bool = False) -> str:
    """hipcc -> paper_2604_06596_amd/libdynlp.so.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [
        hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC", "-pthread",
        # packed-FP32 instruction selection is switched off for all device code
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(_ROOT, "include"), "-I", os.path.join(_HERE, "csrc"),
        "-o", _SO + ".tmp", _SRC,
    ]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr[-4000:])
    os.replace(_SO + ".tmp", _SO)
    return _SO


if __name__ == "__main__":
    print(build(verbose=True))
