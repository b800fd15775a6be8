"""Build libnf4.so (the C-ABI library of include/nf4.h) for gfx950 with hipcc.

In-tree: the library lands next to this file so that it travels with the
source tree.  hipcc cross-compiles without a GPU.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libnf4.so")
SOURCES = ["nf4_api.hip", "nf4_dequant.hip", "nf4_gemv.hip", "nf4_quantize_ref.hip", "nf4_quantize.hip", "nf4_gemm.hip", "nf4_gemm_splitk.hip",
           "nf4_gemv_static.hip", "nf4_gemv_slice.hip", "nf4_gemv_quad.hip"]

# -ffp-contract=off: every FP32 multiply and add is rounded on its own, as the
# format's definition states (FMAs are written explicitly where wanted).
# -packed-fp32-ops is switched off: the kernels use scalar FP32 instructions only.
# -amdgpu-kernarg-preload-count: the first kernel arguments (up to 14 dwords) arrive in the wave's initial scalar
# registers instead of through a scalar load that every wave waits for before its first memory request; firmware
# without the feature runs the compatibility prologue the compiler emits, which loads them as before.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-kernarg-preload-count=14",
         "-Wall", "-Wno-unused-command-line-argument"]


STUDY_SRC = os.path.join(HERE, "study", "codebook_study.hip")
STUDY_BIN = os.path.join(HERE, "study", "codebook_study")


def lib_path() -> str:
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    for name in os.listdir(CSRC):
        if os.path.getmtime(os.path.join(CSRC, name)) > t:
            return True
    return os.path.getmtime(os.path.join(HERE, "..", "include", "nf4.h")) > t


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-shared", "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    build_study(verbose)
    return LIB


def build_study(verbose: bool = False) -> str:
    """The codebook-placement study: a standalone measurement program (not part of libnf4)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + [f for f in FLAGS if f != "-fPIC"] + ["-o", STUDY_BIN, STUDY_SRC]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return STUDY_BIN


if __name__ == "__main__":
    print(build(verbose=True))
