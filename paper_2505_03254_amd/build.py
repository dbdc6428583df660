"""Builds libprom.so (the C-ABI library of HIP kernels for gfx950) in-tree with hipcc.

Run as a script (`python -m paper_2505_03254_amd.build`) or call build().  Object files
go to paper_2505_03254_amd/_build/ and are compiled in parallel.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
BUILD_DIR = os.path.join(_HERE, "_build")
LIB_PATH = os.path.join(_HERE, "libprom.so")
SOURCES = ["prom_host.cpp", "prom_pw.hip", "prom_pw_rows.hip", "prom_pw_big.hip", "prom_pw_gemm.hip", "prom_pw_addsub.hip", "prom_dw.hip", "prom_gconv.hip", "prom_block.hip", "prom_block_planes.hip", "prom_dwproj.hip", "prom_quant.hip", "prom_pw_dynq.hip", "prom_bench.hip"]
PW_MAX_NT = 10  # prom_pw_inst.hip is compiled once per NT = 1..PW_MAX_NT (kMaxNT in prom_pw_stream.h)

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _extra_flags():
    """Extra hipcc flags for a developer build, e.g. PROM_BUILD_FLAGS=-DPROM_TIMELINE."""
    return os.environ.get("PROM_BUILD_FLAGS", "").split()


def _compile(job) -> str:
    src, defines, tag = job
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + tag + ".o")
    cmd = [_hipcc()] + HIPCC_FLAGS + _extra_flags() + defines + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in p.stderr.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    # the heaviest units (large NT) first
    jobs = [("prom_pw_inst.hip", [f"-DPROM_PW_NT={n}"], f"_nt{n}") for n in range(PW_MAX_NT, 0, -1)]
    jobs += [(src, [], "") for src in SOURCES]
    workers = min(os.cpu_count() or 4, 16, len(jobs))
    with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as ex:
        objs = list(ex.map(_compile, jobs))
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    subprocess.check_call(cmd)
    os.replace(tmp, LIB_PATH)
    if verbose:
        print("built", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
