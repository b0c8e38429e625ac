"""Compile the HIP sources of the library for gfx950 into ``libhstu_attn.so`` next to this file.

hipcc cross-compiles without a GPU.  The built library is what the tests, the smoke
check and the benchmark load; rebuild after changing anything under ``csrc/``.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhstu_attn.so")
SOURCES = ["api.hip", "schedule.hip", "attn_core.hip", "attn_fwd_pipe.hip", "gated_norm.hip", "truncate.hip", "pointwise.hip", "gemm.hip", "gemm_tn.hip", "layer.hip", "fp8_gemm.hip", "lbsl.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         # packed fp32 VALU forms are kept off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str, objdir: str, defines=()) -> str:
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *[f"-D{d}" for d in defines], "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError(f"hipcc failed for {src}")
    return obj


def build_library(verbose: bool = False, defines=(), output: str = LIB) -> str:
    """Build the library.  ``defines`` (``NAME=VALUE`` strings) and ``output`` are for measurement builds, which
    bindings pick up through the HSTU_ATTN_LIB environment variable; the default is the product."""
    objdir = os.path.join(HERE, "_build" if not defines else "_build_" + "_".join(d.replace("=", "-") for d in defines))
    os.makedirs(objdir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(lambda s: _compile(s, objdir, defines), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", output, *objs, "-lhipblaslt"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("link failed")
    if verbose:
        print("built", output)
    return output


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--define", action="append", default=[], metavar="NAME=VALUE", help="extra preprocessor definition (measurement builds)")
    ap.add_argument("--output", default=LIB, help="path of the shared library to write")
    ns = ap.parse_args()
    build_library(verbose=True, defines=tuple(ns.define), output=ns.output)
