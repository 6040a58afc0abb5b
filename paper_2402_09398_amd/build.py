"""Builds liblessdec.so (HIP, gfx950) in-tree next to this file."""
from __future__ import annotations

import os
import subprocess
import sys
from pathlib import Path

HERE = Path(__file__).resolve().parent
ROOT = HERE.parent
CSRC = HERE / "csrc"
LIB = HERE / "liblessdec.so"
SOURCES = ["lessdec_api.hip", "lessdec_featmap.hip", "lessdec_mlp.hip", "lessdec_step.hip", "lessdec_wpu.hip",
           "lessdec_prefill.hip", "lessdec_gqa.hip", "lessdec_gqs.hip", "lessdec_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    f"-I{ROOT / 'include'}", f"-I{CSRC}",
]


def build(verbose: bool = True) -> Path:
    """Compile every HIP source into one shared library; always recompiles."""
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    cmd = [HIPCC, *FLAGS, "-o", str(tmp), *[str(CSRC / s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
