"""Build ``libsinglequant.so`` in-tree with hipcc for gfx950 (cross-compiles without a GPU).

    python -m paper_2511_22316_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_CSRC = os.path.join(_HERE, "csrc")
_OUT = os.path.join(_HERE, "libsinglequant.so")

SOURCES = ["sq_rotate_quantize.hip", "sq_rotq_mfma.hip", "sq_w4a4_gemm.hip", "sq_prepare_weights.hip", "sq_build_rotation.hip", "sq_decode_layer.hip", "sq_w4a16_gemm.hip",
           "sq_status.cpp"]

# packed-fp32 VALU forms are switched off for every HIP translation unit of this library
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-inline-asm", "-fno-honor-nans"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every translation unit (in parallel, objects under csrc/_build/) and link the
    shared library.  Always recompiles everything."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(_CSRC, "_build")
    os.makedirs(objdir, exist_ok=True)
    common = [hipcc, *[f for f in FLAGS if f != "-shared"], *extra_flags, "-I", os.path.join(_ROOT, "include"),
              "-I", _CSRC]

    def compile_one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        _run([*common, "-c", "-x", "hip", os.path.join(_CSRC, src), "-o", obj], verbose)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", _OUT, *objs], verbose)
    return _OUT


if __name__ == "__main__":
    print(build(verbose=True))
