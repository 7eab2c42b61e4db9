"""Compiles the HIP/C++ sources under csrc/ into libmgwfbp.so next to this file, and the benchmark's
measurement aid under bench_aid/ into its own shared object there (gfx950 only)."""
from __future__ import annotations

import os
import shutil
import subprocess
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_NAME = "libmgwfbp.so"
SOURCES = ("plan.cpp", "model.cpp", "layout.cpp", "kernels.hip")
AID_DIR = os.path.join(ROOT, "bench_aid")
AID_LIB = os.path.join(AID_DIR, "libmgwfbp_bench_aid.so")

# -ffp-contract=off: the update and the reduction promise one rounding per operation.
# The packed-fp32 feature is switched off for device code: packed single-precision instructions are
# not wanted in these kernels.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def library_path() -> str:
    return os.path.join(HERE, LIB_NAME)


def build_library(out: Optional[str] = None, defines: Optional[Dict[str, object]] = None,
                  verbose: bool = False) -> str:
    """Always recompiles.  `defines` lets a tuning run override MGWFBP_TILE_VECS / MGWFBP_NT."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    out = out or library_path()
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for k, v in (defines or {}).items():
        cmd.append(f"-D{k}={v}")
    cmd += ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{res.stdout}")
    if verbose and res.stdout.strip():
        print(res.stdout)
    return out


def build_bench_aid(verbose: bool = False) -> str:
    """The stream probe and cache scrub that bench.py uses; kept out of libmgwfbp.so on purpose."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", AID_DIR, "-x", "hip", os.path.join(AID_DIR, "stream_probe.hip"), "-o", AID_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{res.stdout}")
    return AID_LIB


if __name__ == "__main__":  # python -m paper_1912_09268_amd.build
    print(build_library(verbose=True))
    print(build_bench_aid(verbose=True))
