"""Build libcbconv.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcbconv.so")
SOURCES = ["cb_detect.hip", "cb_compact.hip", "cb_gather.hip", "cb_gemm.hip", "cb_fused.hip", "cb_fused_f32.hip", "cb_fused_cl.hip",
           "cb_fused_bf16.hip", "cb_update.hip", "cb_metric.hip", "cbconv.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-fast-math", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    noise = "is not a recognized feature for this target"
    for line in r.stderr.splitlines():
        if line.strip() and noise not in line:
            print(line, file=sys.stderr)
    return obj


def build_library(verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    # Link against the HIP runtime that torch itself loads (its bundled libamdhip64.so),
    # so that torch's streams and allocations are valid in this library: two HIP
    # runtimes in one process would not share them.
    import torch
    tlib = os.path.join(os.path.dirname(torch.__file__), "lib")
    if os.path.exists(os.path.join(tlib, "libamdhip64.so")):
        hip_link = ["-L" + tlib, "-l:libamdhip64.so", "-Wl,-rpath," + tlib]
    else:
        rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
        hip_link = ["-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    cmd = ["g++", "-shared", "-fPIC", "-o", LIB, *objs, *hip_link, "-Wl,--no-undefined"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build_library()
