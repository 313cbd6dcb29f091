"""Builds paper_2301_12017_amd/libw4a4.so from csrc/*.hip with hipcc for gfx950.

hipcc cross-compiles without a GPU, so this runs on the build host; the shared
object then travels with the tree.  Flags:
  -ffp-contract=off   the quantizer and epilogue rely on separately rounded fp32
                      operations (codes must be reproducible bit for bit);
  -packed-fp32-ops    feature switched OFF: no v_pk_*_f32 instructions are generated.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libw4a4.so")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "quantize.hip", "epilogue.hip", "gemm.hip", "gemm_generic.hip", "gemm_pipe.hip", "gemm_olay.hip", "gemm_fp6.hip", "gemm_group.hip", "gemm_small.hip", "layernorm.hip", "gemm_w8.hip", "quantize_w8.hip", "strategy.hip", "attention.hip", "probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fhip-fp32-correctly-rounded-divide-sqrt",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    subprocess.run([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
