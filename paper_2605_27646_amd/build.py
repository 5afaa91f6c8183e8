"""Build libhqmq.so (the C-ABI HQMQ library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhqmq.so")

SOURCES = ["hqmq_api.hip", "hqmq_median.hip", "hqmq_search.hip", "hqmq_decode.hip", "hqmq_attend.hip",
           "hqmq_codebook.cpp"]

FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-ffp-contract=off",          # every fused multiply-add in the sources is written explicitly
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 VALU forms
    "-fno-honor-nans",            # inputs are finite by contract; drops NaN-quieting max/min pairs
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",  # MFMA results straight into VGPRs for the VALU epilogue
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"),
    "-I", CSRC,
]


def build(verbose: bool = False, extra: list[str] | None = None, out: str | None = None) -> str:
    """Compile the library to `out` (default: libhqmq.so beside this file)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = out or LIB
    cmd = [hipcc, *FLAGS, *(extra or []), "-o", out, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    lines = [ln for ln in (res.stdout + res.stderr).splitlines()
             if "packed-fp32-ops" not in ln or "error" in ln]
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
    if verbose and lines:
        print("\n".join(lines))
    return out


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
