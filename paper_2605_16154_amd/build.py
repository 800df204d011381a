"""Builds libpcm.so (the C-ABI library of include/pcm.h) and libpcm_measure.so (the stand-alone
matrix-core rate probe of include/pcm_measure.h) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpcm.so")
MEASURE_LIB = os.path.join(PKG, "libpcm_measure.so")
OBJ_DIR = os.path.join(PKG, "_build")

SOURCES = ["runtime.hip", "score.hip", "keep_probs.hip", "sample.hip", "gather.hip",
           "actor_f32.hip", "actor_bf16.hip", "actor_api.hip", "optimizer.hip", "labeler.hip"]
MEASURE_SOURCES = ["measure/mfma_rate.hip"]
# the fp64 tails of the selection stage are specified without fused multiply-add
NO_CONTRACT = {"score.hip", "keep_probs.hip"}

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, src.replace("/", "_").replace(".hip", ".o"))
    cmd = [_hipcc(), *COMMON, "-c", os.path.join(CSRC, src), "-o", obj]
    if src in NO_CONTRACT:
        cmd.insert(1, "-ffp-contract=off")
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(jobs: int = 8) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES + MEASURE_SOURCES))
    for lib, part in ((LIB, objs[:len(SOURCES)]), (MEASURE_LIB, objs[len(SOURCES):])):
        cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *part]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


C_CLIENT_SRC = os.path.join(ROOT, "tests", "c", "gpu_client.cpp")
C_CLIENT = os.path.join(ROOT, "tests", "c", "gpu_client")


def build_c_client() -> str:
    """The torch-free client of the C boundary that tests/test_gpu_c_client.py runs (host code only; it finds
    libpcm.so relative to its own location)."""
    cmd = [_hipcc(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "include"), C_CLIENT_SRC,
           "-o", C_CLIENT, "-L", PKG, "-l:libpcm.so", "-Wl,-rpath,$ORIGIN/../../paper_2605_16154_amd"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the C client failed:\n" + r.stderr)
    return C_CLIENT


if __name__ == "__main__":
    print(build_library())
    print(build_c_client())
