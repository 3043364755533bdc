"""Builds libtokenscale.so (HIP kernels + C ABI) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtokenscale.so")

SOURCES = ["ts_planner.cpp", "ts_policy.cpp", "ts_api.hip", "ts_kernels_append.hip", "ts_kernels_rows.hip",
           "ts_kernels_decode.hip", "ts_kernels_prefill.hip", "ts_kernels_mixed.hip", "ts_calib.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
         # no packed fp32 instructions from the auto-vectoriser
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # IEEE-rounded fp32 division (the fp8 quantiser must match a single rounding)
         "-fhip-fp32-correctly-rounded-divide-sqrt",
         # keep MFMA accumulators in VGPRs so that the softmax rescale needs no AGPR copies
         "-mllvm", "-amdgpu-mfma-vgpr-form",
         # the LDS-copy asm statements name m0 as clobbered (so the compiler knows its own m0 values are gone);
         # the backend remarks that m0 is a reserved register, which is the point
         "-Wno-inline-asm",
         "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
