"""Builds libhexa_moe.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhexa_moe.so")
SOURCES = ["api.hip", "index.hip", "elementwise.hip", "f32_path.hip", "gemm_bf16.hip", "probe.hip", "route.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.check_call(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build_library(jobs: int = 7) -> str:
    """Compile every translation unit and link the shared library.  Always rebuilds."""
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build_library())
