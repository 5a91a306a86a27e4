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


def _filter(stderr: str) -> str:
    return "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l)


def build_hip(verbose: bool = False) -> str:
    """Compile every source to an object file (in parallel), then link the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-I" + os.path.join(_ROOT, "include"), "-I" + _CSRC,
             # keep the compiler from forming packed fp32 instructions
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        res = subprocess.run(["hipcc"] + flags + ["-c", os.path.join(_CSRC, src), "-o", obj],
                             capture_output=True, text=True)
        return src, obj, res

    with ThreadPoolExecutor(max_workers=min(8, len(HIP_SOURCES))) as pool:
        results = list(pool.map(compile_one, HIP_SOURCES))
    failed = False
    for src, _, res in results:
        err = _filter(res.stderr)
        if (verbose or res.returncode) and err.strip():
            sys.stderr.write(f"---- {src}\n{err}\n")
        failed = failed or res.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [o for _, o, _ in results],
                         capture_output=True, text=True)
    if res.returncode:
        sys.stderr.write(_filter(res.stderr) + "\n")
        raise RuntimeError("hipcc link failed")
    return LIB


def build_all(verbose: bool = False):
    from . import synth
    synth.build_synth(force=True)
    return build_hip(verbose)


if __name__ == "__main__":
    print(build_all(verbose=True))
