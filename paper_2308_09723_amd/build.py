"""Builds libfq.so for gfx950 with hipcc (cross-compiles without a GPU).

Every translation unit is compiled to an object file in parallel (the nine product-kernel
instantiations dominate the build time), then linked into paper_2308_09723_amd/libfq.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libfq.so")
SOURCES = [
    "fq_api.hip",
    "fq_quantize.hip",
    "fq_gemm.hip",
    "fq_gemm_f16_4.hip",
    "fq_gemm_f16_8.hip",
    "fq_gemm_bf16_4.hip",
    "fq_gemm_bf16_8.hip",
    "fq_gemm_bf16s_4.hip",
    "fq_gemm_bf16s_8.hip",
    "fq_gemm_f16_3.hip",
    "fq_gemm_bf16_3.hip",
    "fq_gemm_bf16s_3.hip",
]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    # correctly rounded binary32 division and no value-changing math: the quantiser is bit-exact
    "-fno-fast-math",
    "-ffp-contract=off",
    # packed-fp32 instruction forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    return res.returncode, out


def build_lib(verbose: bool = True, jobs: int | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    jobs = jobs or min(len(SOURCES), len(os.sched_getaffinity(0)), 8)

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        rc, out = _run(cmd)
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    rc, out = _run(cmd)
    if rc != 0:
        raise RuntimeError("link failed:\n" + out)
    return LIB_PATH


if __name__ == "__main__":
    build_lib()
    sys.exit(0)
