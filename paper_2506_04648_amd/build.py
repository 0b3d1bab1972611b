"""Builds libfps.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
SOURCES = ("fps_host.cpp", "fps_layout.hip", "fps_quantize.hip", "fps_attn.hip", "fps_issue_mix.hip")
OUT = os.path.join(_HERE, "libfps.so")


def build_lib(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"),
           # packed fp32 instructions stay off (they are generated from ordinary float code otherwise)
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # MFMA results stay in architectural VGPRs: the softmax VALU code reads them directly
           # instead of through v_accvgpr moves
           "-mllvm", "-amdgpu-mfma-vgpr-form",
           # no NaN ever enters the kernels (inputs are finite, masked scores are -inf, never inf-inf):
           # lets fmax/fmin compile without the canonicalising v_max(x,x) in front of every operand
           "-fno-honor-nans",
           "-o", OUT] + os.environ.get("FPS_EXTRA_HIPCC_FLAGS", "").split() \
          + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libfps.so")
    return OUT
