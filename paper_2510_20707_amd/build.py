"""Builds libmixkv.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2510_20707_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmixkv.so")
SOURCES = ["mixkv_api.hip", "mixkv_stream.hip", "mixkv_mixsel.hip", "mixkv_select.hip", "mixkv_analysis.hip", "mixkv_decode.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-amdgpu-mfma-vgpr-form",     # MFMA results land in VGPRs: the VALU reads them directly
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build_lib(verbose: bool = False, extra=()) -> str:
    cmd = [HIPCC, *FLAGS, *extra, "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed building libmixkv.so")
    if verbose:
        # the host pass says it does not know the packed-fp32 feature; that warning is expected
        noise = "is not a recognized feature for this target"
        sys.stderr.write("\n".join(l for l in r.stderr.splitlines() if noise not in l) + "\n")
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
