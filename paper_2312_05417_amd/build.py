"""Builds libespn.so (the C-ABI library) for gfx950 with hipcc, in-tree, next to the binding."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libespn.so")
SOURCES = [os.path.join(CSRC, "espn.hip")]
# the benchmark's measuring sticks (a plain read, a plain copy): a library of their own, not part of the product ABI
PROBE_LIB = os.path.join(HERE, "libespn_benchprobe.so")
PROBE_SOURCES = [os.path.join(CSRC, "bench_probe.hip")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    "-fno-gpu-sanitize", "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # device code only: inputs are finite by contract, so max() chains need no NaN quieting
    # (v_max3_f32 instead of three v_max_f32 per operand pair); NaN tests in the kernels look at bits
    "-Xarch_device", "-fno-honor-nans",
    # MFMA results straight into VGPRs (no v_accvgpr_read before the VALU maximum)
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
]


def hipcc() -> str:
    cand = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "bin", "hipcc")
    return cand if os.path.exists(cand) else "hipcc"


def _compile(lib, sources, verbose, extra_flags) -> str:
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-o", tmp, *sources]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


def build_library(verbose: bool = True, extra_flags=()) -> str:
    _compile(PROBE_LIB, PROBE_SOURCES, verbose, extra_flags)
    return _compile(LIB, SOURCES, verbose, extra_flags)


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
