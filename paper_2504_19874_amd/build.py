"""Builds libturboquant.so (HIP, gfx950 only) next to this file.

    python -m paper_2504_19874_amd.build

hipcc cross-compiles without a GPU.  The flags switch off packed-fp32 code
generation, as the target boxes require.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libturboquant.so")
PROBE_LIB = os.path.join(HERE, "libtqprobe.so")  # measurement aid of bench_kernels, not part of the library
OBJ = os.path.join(HERE, "_build")

SOURCES = ["tq_api.hip", "tq_gemm.hip", "tq_d128.hip", "tq_d128_small.hip", "tq_d128_small_dq.hip", "tq_score_small.hip", "tq_score_i8.hip", "tq_score_i8_128.hip", "tq_score_i8_split.hip", "tq_score_bf3.hip", "tq_d128_bf3.hip", "tq_q128_bf3.hip", "tq_stage.hip", "tq_attend.hip", "tq_attend_128.hip", "tq_attend_128_v1.hip", "tq_attend_128_v2.hip", "tq_attend_128_v3.hip", "tq_attend_128_v4.hip", "tq_attend_128_p0.hip", "tq_attend_128_p1.hip", "tq_attend_128_p2.hip", "tq_attend_128_s1.hip", "tq_attend_128_s2.hip", "tq_topk.hip",
           "tq_codebook.cpp", "tq_rotation.cpp", "tq_entropy.cpp"]
HIP_FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *HIP_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    if src.endswith(".cpp"):
        cmd = ["hipcc", "-O2", "-fPIC", "-std=c++17", "-x", "c++", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    return obj


def build_library(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    cmd = ["hipcc", *HIP_FLAGS, "-shared", os.path.join(CSRC, "probe_intake.hip"), "-o", PROBE_LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
