"""Compile the HIP library for gfx950 (cross-compiles without a GPU).

    python -m paper_2410_01699_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsjd_hip.so")

# packed-fp32 instructions are switched off for every device compile (a known hazard on the test machines)
COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          # leading kernel arguments arrive in SGPRs with the dispatch (no scalar load in front of a
          # kernel's first memory accesses); kernels keep a fallback prologue for firmware without it
          "-mllvm", "-amdgpu-kernarg-preload-count=16",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# the sampling file needs every fp32 operation rounded separately (bit-exact contract)
PER_FILE = {"sjd_sample.hip": ["-ffp-contract=off"]}
SOURCES = ["sjd_api.hip", "sjd_gemm.hip", "sjd_gemm_bf16.hip", "sjd_gemm_wide.hip", "sjd_layers.hip", "sjd_attention.hip", "sjd_sample.hip"]


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = ["hipcc", *COMMON, *PER_FILE.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        return src, obj, r

    with ThreadPoolExecutor(len(SOURCES)) as ex:
        results = list(ex.map(compile_one, SOURCES))
    objs = []
    for src, obj, r in results:
        noise = "unknown and unsupported by the target"
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l and "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        objs.append(obj)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
