"""Build the HIP library in-tree: paper_2312_08583_amd/libfp6_linear.so (gfx950 only)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfp6_linear.so")
SOURCES = ["fp6_abi.hip", "fp6_pack.hip", "fp6_decode.hip", "fp6_gemm.hip", "fp6_gemm_variants.hip", "fp6_gemm_bf16.hip", "fp6_probes.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         # packed-fp32 VALU forms are switched off for every kernel of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(verbose: bool = False, extra_flags=(), lib: str = LIB, tag: str = "") -> str:
    """Compile every source and link `lib`.  extra_flags / tag are for tuning builds (-D switches)."""
    os.makedirs(OBJ, exist_ok=True)

    def _compile(src: str) -> str:
        obj = os.path.join(OBJ, os.path.splitext(src)[0] + tag + ".o")
        subprocess.run(["hipcc", *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
        return obj

    with ThreadPoolExecutor(max_workers=7) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(verbose=True)
