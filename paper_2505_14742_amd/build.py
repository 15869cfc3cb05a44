"""Build libquaff.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libquaff.so")

SOURCES = ["quaff_api.cpp", "quaff_prepare.hip", "quaff_scale.hip", "quaff_quant.hip", "quaff_lora.hip", "quaff_lora_stream.hip", "quaff_quant_lora.hip", "quaff_fwd_step.hip", "quaff_fwd_prep.hip", "quaff_what_quant.hip", "quaff_lora_grad.hip", "quaff_outlier_grad.hip", "quaff_calib.hip",
           "quaff_gemm.hip", "quaff_profile.cpp", "quaff_microbench.hip"]

# -ffp-contract=off: the quantizer's fp32 operation sequence is part of the arithmetic contract (no fused
# multiply-add unless written explicitly); correctly rounded fp32 divide and sqrt for the same reason.
HIPFLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip", "-ffp-contract=off",
            "-fhip-fp32-correctly-rounded-divide-sqrt", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    subprocess.check_call(["hipcc", *HIPFLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
