"""Builds the HIP library (gfx950) in-tree: paper_1804_10574_amd/libddg.so, and the stand-alone
measuring tool paper_1804_10574_amd/ddg_peaks (attained HBM bandwidth and MFMA rates)."""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libddg.so")
PEAKS = os.path.join(HERE, "ddg_peaks")

SOURCES = ["kernels_conv.hip", "kernels_conv_tiled.hip", "kernels_conv_tiled_f32.hip", "kernels_conv_wide.hip", "kernels_wgrad.hip", "kernels_wgrad_tiled.hip", "kernels_wgrad_wide.hip", "kernels_elem.hip", "ddg_scratch.hip", "ddg_module.cpp", "ddg_pipeline.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed on " + src)
    warn = [l for l in (r.stdout + r.stderr).splitlines()
            if l.strip() and "packed-fp32-ops" not in l]
    if warn:
        sys.stderr.write("\n".join(warn) + "\n")
    return obj


def build_library(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    r = subprocess.run([HIPCC] + FLAGS + [os.path.join(CSRC, "peaks_main.hip"), "-o", PEAKS], capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed on peaks_main.hip")
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library()
