"""Builds libhexa_moe.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhexa_moe.so")
SOURCES = ["api.hip", "index.hip", "elementwise.hip", "f32_path.hip", "gemm_bf16.hip", "probe.hip", "route.hip",
           "bench_support.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


# The contraction kernels count their own direct-to-LDS loads in vmcnt; a register spill inside
# their K loop would add vector-memory operations the count does not know about.  So the build
# refuses a gemm_bf16.hip whose kernels use any scratch memory at all.  (About 1 KB of scratch per
# lane in one instantiation means its K loop was left rolled: LLVM ignores "#pragma unroll" past a
# size threshold, -mllvm -pragma-unroll-threshold=N, and the accumulator and fragment arrays are
# then indexed dynamically and live in scratch.)
NO_SCRATCH = {"gemm_bf16.hip"}


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    if src not in NO_SCRATCH:
        subprocess.check_call(cmd)
        return obj
    res = subprocess.run(cmd + ["-Rpass-analysis=kernel-resource-usage"], stderr=subprocess.PIPE, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{res.stderr}")
    name, bad = None, []
    for line in res.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and int(m.group(1)) > 0 and name and "gemm_bf16" in name:
            bad.append((name, int(m.group(1))))
    if bad:
        raise RuntimeError(f"{src}: kernels spill registers (scratch bytes per lane): {bad}")
    return obj


def build_library(jobs: int = 7) -> str:
    """Compile every translation unit and link the shared library.  Always rebuilds."""
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


# ---- host-code sanitizer build (CPU-side checks only; the device code is compiled as usual) ----
SAN_LIB = os.path.join(HERE, "libhexa_moe_asan.so")
SAN_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined"]


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer runtime that the sanitized library needs preloaded."""
    out = subprocess.check_output(["/opt/rocm/llvm/bin/clang++", "-print-file-name=libclang_rt.asan-x86_64.so"],
                                  text=True).strip()
    if not os.path.exists(out):
        raise RuntimeError("clang's AddressSanitizer runtime was not found")
    return out


def build_sanitized_library(jobs: int = 7) -> str:
    """libhexa_moe_asan.so: the same sources with AddressSanitizer and UndefinedBehaviorSanitizer on the
    host code (argument checks, workspace layout, launch set-up).  tests/test_sanitizers.py runs the
    host-only ABI tests against it; GPU sanitizers are not used."""
    def one(src: str) -> str:
        obj = os.path.join(CSRC, src.replace(".hip", ".asan.o"))
        flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g", "-fno-omit-frame-pointer"]
        subprocess.check_call(["hipcc", *flags, *SAN_HOST, "-c", os.path.join(CSRC, src), "-o", obj])
        return obj
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(one, SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined",
                           "-shared-libsan", "-o", SAN_LIB, *objs])
    return SAN_LIB


if __name__ == "__main__":
    import sys
    print(build_sanitized_library() if "--sanitize" in sys.argv[1:] else build_library())
