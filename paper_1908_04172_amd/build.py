"""Builds the C-ABI library (hipcc, gfx950 only) in-tree: paper_1908_04172_amd/libhe_mi355x.so."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhe_mi355x.so")
SOURCES = ["he_api.hip", "he_mac.hip", "he_ntt.hip", "he_ubench.hip", "he_encode.hip", "he_packed32.hip", "he_relin.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the butterfly loops must unroll completely (register arrays are indexed by their counters)
         "-mllvm", "-pragma-unroll-threshold=1000000"]


def _compile(src: str, extra) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.check_call(["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(extra_flags=()) -> str:
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        objs = list(pool.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(sys.argv[1:]))
