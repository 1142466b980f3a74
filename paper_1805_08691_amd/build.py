"""Compiles the HIP sources in csrc/ for gfx950 into libq8conv.so next to this file.

Run as ``python -m paper_1805_08691_amd.build``.  Flags: no fused multiply-add
(-ffp-contract=off, the epilogue's op order is part of the result), packed-fp32
instructions disabled, correctly rounded fp32 division and square root (hipcc default).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.environ.get("Q8_OBJ_DIR") or os.path.join(HERE, "_build")
LIB = os.environ.get("Q8_LIB_OUT") or os.path.join(HERE, "libq8conv.so")
SOURCES = ["q8_conv_ring.hip", "q8_conv_ring_ext.hip", "q8_conv_ring_pair.hip", "q8_conv_chain.hip",
           "q8_conv_halo.hip", "q8_conv_dual.hip", "q8_conv_pw.hip", "q8_conv_split.hip", "q8_conv_p3.hip", "q8_conv_stem.hip",
           "q8_conv.hip", "q8_conv_reg.hip", "q8_elementwise.hip", "q8_helpers.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
EXTRA = os.environ.get("Q8_EXTRA_FLAGS", "").split()
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fhip-fp32-correctly-rounded-divide-sqrt",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA accumulators live in ordinary VGPRs (the epilogue reads them with vector
         # instructions): no copies between VGPRs and AGPRs
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         "-Wall", "-Wno-unused-function",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    subprocess.check_call([HIPCC, *FLAGS, *EXTRA, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
