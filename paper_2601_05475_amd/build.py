"""Compile the HIP library (gfx950) and the host-side input generator, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_CSRC = os.path.join(_HERE, "csrc")
HIP_SOURCES = ["runtime.hip", "ops.hip", "kernels_basic.hip", "kernels_mfma.hip", "kernels_gemm.hip", "kernels_attn.hip",
               "kernels_prefill_attn.hip", "search_host.hip"]
LIB = os.path.join(_HERE, "libmaxcode_mi355x.so")


def build_hip(verbose: bool = False) -> str:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(_ROOT, "include"), "-I" + _CSRC,
           # keep the compiler from forming packed fp32 instructions
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", LIB] + [os.path.join(_CSRC, s) for s in HIP_SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if verbose or res.returncode:
        sys.stderr.write(err + "\n")
    if res.returncode:
        raise RuntimeError("hipcc failed")
    return LIB


def build_all(verbose: bool = False):
    from . import synth
    synth.build_synth(force=True)
    return build_hip(verbose)


if __name__ == "__main__":
    print(build_all(verbose=True))
