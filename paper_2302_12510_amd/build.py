"""Builds libdybit.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdybit.so")
# (source, object stem, extra flags): the tiled kernels are compiled once per weight format
SOURCES = [
    ("host.cpp", "host", []),
    ("quantize.hip", "quantize", []),
    ("metric.hip", "metric", []),
    ("dwconv.hip", "dwconv", []),
    ("pool.hip", "pool", []),
    ("search.cpp", "search", []),
    ("gemm.hip", "gemm", []),
    ("gemm_dispatch.cpp", "gemm_dispatch", []),
    ("gemm_fast.hip", "gemm_fast_w4", ["-DDYBIT_FAST_W=0"]),
    ("gemm_fast.hip", "gemm_fast_w8", ["-DDYBIT_FAST_W=2"]),
    ("gemm_fast.hip", "gemm_fast_w6", ["-DDYBIT_FAST_W=4"]),
    ("gemm_fast.hip", "gemm_fast_w2", ["-DDYBIT_FAST_W=6"]),
    ("gemm_mid.hip", "gemm_mid_w4", ["-DDYBIT_MID_W=0"]),
    ("gemm_mid.hip", "gemm_mid_w8", ["-DDYBIT_MID_W=2"]),
    ("gemm_mid.hip", "gemm_mid_w6", ["-DDYBIT_MID_W=4"]),
    ("gemm_mid.hip", "gemm_mid_w2", ["-DDYBIT_MID_W=6"]),
    ("gemm_f8.hip", "gemm_f8_w4", ["-DDYBIT_F8_W=0"]),
    ("gemm_f8.hip", "gemm_f8_w2", ["-DDYBIT_F8_W=6"]),
    ("gemm_ws.hip", "gemm_ws_w4", ["-DDYBIT_WS_W=0"]),
    ("gemm_ws.hip", "gemm_ws_w8", ["-DDYBIT_WS_W=2"]),
    ("gemm_ws.hip", "gemm_ws_w6", ["-DDYBIT_WS_W=4"]),
    ("gemm_ws.hip", "gemm_ws_w2", ["-DDYBIT_WS_W=6"]),
    # write-back builds of the same kernels (epilogue also encodes the results as DyBit codes)
    ("gemm.hip", "gemm_wb_a2", ["-DDYBIT_WB=1", "-DDYBIT_GEN_A=2"]),
    ("gemm.hip", "gemm_wb_a4", ["-DDYBIT_WB=1", "-DDYBIT_GEN_A=4"]),
    ("gemm.hip", "gemm_wb_a6", ["-DDYBIT_WB=1", "-DDYBIT_GEN_A=6"]),
    ("gemm.hip", "gemm_wb_a8", ["-DDYBIT_WB=1", "-DDYBIT_GEN_A=8"]),
    ("gemm_fast.hip", "gemm_fast_w4_wb", ["-DDYBIT_FAST_W=0", "-DDYBIT_WB=1"]),
    ("gemm_fast.hip", "gemm_fast_w8_wb", ["-DDYBIT_FAST_W=2", "-DDYBIT_WB=1"]),
    ("gemm_fast.hip", "gemm_fast_w6_wb", ["-DDYBIT_FAST_W=4", "-DDYBIT_WB=1"]),
    ("gemm_fast.hip", "gemm_fast_w2_wb", ["-DDYBIT_FAST_W=6", "-DDYBIT_WB=1"]),
    ("gemm_mid.hip", "gemm_mid_w4_wb", ["-DDYBIT_MID_W=0", "-DDYBIT_WB=1"]),
    ("gemm_mid.hip", "gemm_mid_w8_wb", ["-DDYBIT_MID_W=2", "-DDYBIT_WB=1"]),
    ("gemm_mid.hip", "gemm_mid_w6_wb", ["-DDYBIT_MID_W=4", "-DDYBIT_WB=1"]),
    ("gemm_mid.hip", "gemm_mid_w2_wb", ["-DDYBIT_MID_W=6", "-DDYBIT_WB=1"]),
    ("gemm_f8.hip", "gemm_f8_w4_wb", ["-DDYBIT_F8_W=0", "-DDYBIT_WB=1"]),
    ("gemm_f8.hip", "gemm_f8_w2_wb", ["-DDYBIT_F8_W=6", "-DDYBIT_WB=1"]),
    ("gemm_ws.hip", "gemm_ws_w4_wb", ["-DDYBIT_WS_W=0", "-DDYBIT_WB=1"]),
    ("gemm_ws.hip", "gemm_ws_w8_wb", ["-DDYBIT_WS_W=2", "-DDYBIT_WB=1"]),
    ("gemm_ws.hip", "gemm_ws_w6_wb", ["-DDYBIT_WS_W=4", "-DDYBIT_WB=1"]),
    ("gemm_ws.hip", "gemm_ws_w2_wb", ["-DDYBIT_WS_W=6", "-DDYBIT_WB=1"]),
    ("diag.hip", "diag", []),
]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(item) -> str:
    src, stem, extra = item
    obj = os.path.join(CSRC, stem + ".o")
    cmd = [_hipcc(), *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in p.stderr.splitlines() if "not a recognized feature" not in l)
    if p.returncode:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        print(err)
    return obj


# Longest compilations first, so that the pool's last jobs are short ones.
_ORDER = ("gemm", "gemm_wb", "gemm_mid", "gemm_ws", "gemm_f8", "gemm_fast", "quantize")


def _rank(item) -> int:
    stem = item[1]
    for i, prefix in enumerate(_ORDER):
        if stem == prefix or (i >= 1 and stem.startswith(prefix)):
            return i
    return len(_ORDER)


def build(verbose: bool = True) -> str:
    jobs = sorted(SOURCES, key=_rank)
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 8)) as ex:
        objs = list(ex.map(_compile, jobs))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode:
        raise RuntimeError("link failed:\n" + p.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
