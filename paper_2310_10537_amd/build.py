"""Compile the HIP sources for gfx950 into paper_2310_10537_amd/libmx.so.

    python -m paper_2310_10537_amd.build

hipcc cross-compiles without a GPU.  Object files go to csrc/_build/ (ignored
by git); the shared library stays in-tree next to this file.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libmx.so")
SOURCES = ["mx_api.hip", "mx_pattern.hip", "mx_cast.hip", "mx_cast_3d.hip", "mx_cast_fast.hip", "mx_cast_dual.hip", "mx_dequant.hip", "mx_dequant_3d.hip", "mx_gemm.hip", "mx_gemm_int8.hip", "mx_gemm_skinny.hip", "mx_gemm_tile_a8.hip",
           "mx_gemm_tile_a6.hip", "mx_gemm_tile_a4.hip", "mx_gemm_tile16_a8.hip", "mx_gemm_tile8_a6.hip", "mx_gemm_tile8_a4.hip", "mx_gemm_probe.hip", "mx_gemm_tileh_a8.hip", "mx_gemm_tileh_a6.hip", "mx_gemm_tileh_a4.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    subprocess.check_call(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build() -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build())
    sys.exit(0)
