"""Builds the C-ABI shared library from ``csrc/`` with hipcc for gfx950.

Run as ``python -m paper_1312_5853_amd.build``; the library lands next to this
file as ``libconvnet_hotpath.so`` (kept out of version control).
"""
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "convnet_hotpath.hip")
LIB = os.path.join(_HERE, "libconvnet_hotpath.so")
CEILING_SRC = os.path.join(_HERE, "csrc", "mfma_ceiling.hip")
CEILING_EXE = os.path.join(_HERE, "mfma_ceiling")
DEPS = [SRC] + [os.path.join(_HERE, "csrc", h) for h in (
    "plan.h", "fastdiv.h", "device_common.h", "conv_colgemm_kernels.h", "conv_bf16_dma_kernels.h", "conv_wgrad_rows_kernels.h",
    "conv_wgrad_kernels.h", "fc_kernels.h",
    "glue_kernels.h")] + [os.path.join(os.path.dirname(_HERE), "include", "convnet_hotpath.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-Wall",
    # no packed-fp32 instruction selection
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in DEPS)


def build(verbose=False):
    """Compile unconditionally."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if verbose or res.returncode != 0:
        sys.stderr.write(err + "\n")
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    # the stand-alone MFMA ceiling probe (no inputs, prints TFLOP/s)
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-o", CEILING_EXE, CEILING_SRC],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
