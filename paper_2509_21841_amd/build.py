"""Builds libzeppelin_attn.so and the bench-side libzeppelin_bench.so (HIP, gfx950) in-tree with hipcc. Usage: python -m paper_2509_21841_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libzeppelin_attn.so")
BENCH_LIB = os.path.join(HERE, "libzeppelin_bench.so")   # measurement aid: the MFMA rate probe, nothing of the engine
BENCH_SOURCES = ["mfma_probe.hip"]
SOURCES = ["zp_api.hip", "zp_noalloc.hip", "attn_fwd.hip", "attn_bwd.hip", "lse_merge.hip", "remap.hip", "zp_partition.cpp", "zp_remap_plan.cpp"]
# packed-fp32 VALU forms are switched off on purpose for this target
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         # keep MFMA results in ordinary VGPRs where possible: avoids accumulator-register copy storms
         "-mllvm", "-amdgpu-mfma-vgpr-form=1"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _filter(text: str) -> str:
    keep = [l for l in text.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    return "\n".join(keep)


def build(verbose: bool = False) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        r = subprocess.run([hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        msg = _filter(r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{msg}")
        if verbose and msg:
            print(msg)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES + BENCH_SOURCES))
    for lib, lib_objs in ((LIB, objs[:len(SOURCES)]), (BENCH_LIB, objs[len(SOURCES):])):
        r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *lib_objs], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + _filter(r.stdout + r.stderr))
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
