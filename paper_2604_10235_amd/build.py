"""Builds libcodecomp.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcodecomp.so")
PEAKS_LIB = os.path.join(HERE, "libcodecomp_peaks.so")      # measurement only: what the GPU sustains
PEAKS_SOURCES = ["peaks.hip", "pass_model.hip"]
ABI_DEMO = os.path.join(HERE, "abi_demo.exe")                # csrc/abi_demo.c: the C ABI used from plain C
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
# the heavy translation units (the MFMA passes, one per head_dim and key type) first: they run side by side
SOURCES = ["score_pass_d128_bf16.hip", "score_pass_d128_fp8.hip", "score_pass_d64_bf16.hip", "score_pass_d64_fp8.hip",
           "api.hip", "score.hip", "select.hip", "gather.hip", "structure.hip", "static_scratch.hip"]
# packed fp32 VALU ops are switched off on purpose (device pass only; the host pass ignores it)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"),
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed on " + src)
    return obj


def build_library(verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 4)) as ex:
        objs = list(ex.map(_compile, SOURCES + PEAKS_SOURCES))
    n = len(SOURCES)
    for lib, members in ((LIB, objs[:n]), (PEAKS_LIB, objs[n:])):
        r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *members, "-o", lib],
                           capture_output=True, text=True)
        if r.returncode != 0:
            sys.stderr.write(r.stdout + r.stderr)
            raise RuntimeError("link failed")
    # a C99 program that uses the library through its C ABI alone (tests/test_gpu_parity.py runs it on the GPU)
    r = subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROCM, "include"),
                        "-I", os.path.join(os.path.dirname(HERE), "include"), os.path.join(CSRC, "abi_demo.c"), "-o", ABI_DEMO,
                        "-L", HERE, "-l:libcodecomp.so", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
                        "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(ROCM, "lib")], capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("building abi_demo failed")
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library()
