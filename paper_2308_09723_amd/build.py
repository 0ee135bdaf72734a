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
    "fq_w4a8.hip",
    "fq_probe.hip",
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
    # per-kernel register / scratch figures as compiler remarks (parsed below into _build/resources.txt)
    "-Rpass-analysis=kernel-resource-usage",
]

# Kernel instantiations on the timed paths that must not spill registers to scratch memory: a spill puts
# scratch traffic into their inner loops and moves with the compiler version.  The build fails if one does.
# (template arguments as in csrc/fq_gemm_kernels.h)
NO_SPILL = [
    "fq_gemm_skinny_kernel<0, 4, 3, 2, 1, 12, 1>",     # decode, fp16 int4 g >= 128: QKV / FC1 / FC2 / out-proj at M = 1
    "fq_gemm_skinny_kernel<0, 4, 1, 4, 1, 12, 1>",     # out-proj at M = 8
    "fq_gemm_mma_kernel<0, 4, 8, 3, 8, 1, false, 2, false, 1>",   # prefill, fp16
    "fq_gemm_mma_kernel<3, 4, 8, 3, 8, 1, false, 2, false, 1>",   # prefill, bf16 on the fp16 matrix path
    "fq_gemm_mma_kernel<0, 4, 2, 3, 4, 1, false, 2, true, 1>",    # M = 32, fp16, post-scaled
]


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    return res.returncode, out


def _parse_resources(text):
    """[(mangled name, vgprs, agprs, scratch bytes per lane, spilled vgprs, waves per SIMD)] from the
    kernel-resource-usage remarks of one compilation."""
    import re

    rows = []
    for blk in re.split(r"remark: Function Name: ", text)[1:]:
        def num(key):
            m = re.search(key + r": (\d+)", blk)
            return int(m.group(1)) if m else -1
        rows.append((blk.split(" ")[0], num("VGPRs"), num("AGPRs"), num(r"ScratchSize \[bytes/lane\]"),
                     num("VGPRs Spill"), num(r"Occupancy \[waves/SIMD\]")))
    return rows


def _strip_remarks(text):
    """Compiler output without the resource remarks (three lines each: remark, source line, caret)."""
    lines = text.splitlines()
    keep, skip = [], 0
    for ln in lines:
        if skip:
            skip -= 1
            continue
        if "[-Rpass-analysis=kernel-resource-usage]" in ln:
            skip = 2 if "Function Name" in ln else 0
            continue
        keep.append(ln)
    return "\n".join(keep)


def _resource_report(rows, verbose):
    """Writes _build/resources.txt, prints the kernels that spill, fails on a spill in NO_SPILL."""
    import shutil

    names = [r[0] for r in rows]
    filt = shutil.which("c++filt")
    if filt and names:
        dem = subprocess.run([filt] + names, stdout=subprocess.PIPE, text=True).stdout.splitlines()
    else:
        dem = names
    table = []
    for d, r in zip(dem, rows):
        short = d.replace("(anonymous namespace)::", "").split("(")[0].replace("void ", "").replace("fqk::", "")
        table.append((short,) + r[1:])
    table.sort()
    with open(os.path.join(OBJ_DIR, "resources.txt"), "w") as f:
        f.write("kernel | VGPRs | AGPRs | scratch bytes/lane | spilled VGPRs | waves/SIMD\n")
        for t in table:
            f.write(" | ".join(str(x) for x in t) + "\n")
    spilling = [t for t in table if t[4] > 0 or t[3] > 0]
    if verbose:
        print(f"{len(table)} kernels compiled, {len(spilling)} use scratch memory (see _build/resources.txt):")
        for t in spilling:
            print(f"  {t[0]}: {t[4]} spilled VGPRs, {t[3]} B/lane of scratch, {t[1]} VGPRs, {t[5]} waves/SIMD")
    bad = [t for t in spilling if t[0] in NO_SPILL]
    missing = [k for k in NO_SPILL if filt and k not in {t[0] for t in table}]
    if bad:
        raise RuntimeError("register spills in kernels that must not spill: " + ", ".join(t[0] for t in bad))
    if missing:
        raise RuntimeError("NO_SPILL names kernels that were not compiled: " + ", ".join(missing))


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
            raise RuntimeError(f"hipcc failed on {src}:\n{_strip_remarks(out)}")
        rest = _strip_remarks(out)
        if verbose and rest.strip():
            print(rest)
        return obj, _parse_resources(out)

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(compile_one, SOURCES))
    objs = [r[0] for r in results]
    _resource_report([row for r in results for row in r[1]], verbose)
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
