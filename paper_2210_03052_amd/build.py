"""Builds libbt.so (the C-ABI HIP library) and libbt_peaks.so (measurement-only kernels: the two peak probes
behind `bench.py --peaks` and the unfused element-wise baselines behind `bench.py --sweep`) in-tree with
hipcc for gfx950.

    python -m paper_2210_03052_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.environ.get("BT_LIB_OUT") or os.path.join(PKG, "libbt.so")   # BT_LIB_OUT: build a variant elsewhere
SOURCES = ["offsets.hip", "gemm.hip", "layernorm.hip", "mha.hip", "layer.hip"]
PEAKS_LIB = os.path.join(PKG, "libbt_peaks.so")
PEAKS_SOURCES = ["peaks.hip", "unfused.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=default",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the first kernel arguments arrive in SGPRs at wave launch instead of through a scalar load at the top of
    # every kernel (the kernels order their arguments by first use); code for the other case is kept in front
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Per-file extras.  The attention kernel runs VALU softmax directly on MFMA results: keep MFMA
# operands and results in VGPRs so that no v_accvgpr_read/write copies sit in its inner loop.
EXTRA_FLAGS = {"mha.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _compile(src: str) -> str:
    obj = os.path.join(PKG, "_build", src.replace(".hip", ".o"))
    os.makedirs(os.path.dirname(obj), exist_ok=True)
    cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build_library(verbose: bool = True) -> str:
    """Compile every HIP source and link libbt.so; always recompiles."""
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + len(PEAKS_SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES + PEAKS_SOURCES))
    for lib, members in ((LIB, objs[:len(SOURCES)]), (PEAKS_LIB, objs[len(SOURCES):])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *members]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
        if verbose:
            print(f"built {lib}")
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
