"""Builds the HIP library in-tree (libssd_mi355x.so next to this file)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libssd_mi355x.so")
MEASURE_LIB = os.path.join(HERE, "libssd_measure.so")      # measurement kernels only, not part of the product
SOURCES = ["kernels_mfma.hip", "kernels_mfma_f32.hip", "gemm_f32_wn3.hip", "gemm_f32_wn2.hip", "gemm_f32_wn4.hip",
           "gemm_swiglu_wn3.hip", "gemm_swiglu_wn4.hip", "gemm_lmhead_wn4.hip", "ssd_api.hip", "kernels_plain.hip"]
MEASURE_SOURCES = ["measure.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result"]


def _compile(src: str) -> str:
    obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
    os.makedirs(os.path.dirname(obj), exist_ok=True)
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build(verbose: bool = False) -> str:
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES + MEASURE_SOURCES))
    for lib, ob in ((LIB, objs[:len(SOURCES)]), (MEASURE_LIB, objs[len(SOURCES):])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *ob, "-o", lib]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
        if verbose:
            print("built", lib)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
