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
# refuses a gemm_bf16.hip whose kernels use any scratch memory at all.  It also refuses scalar
# register spills: a spilled scalar comes back through v_readlane, and a vector-memory instruction
# must not read a scalar register within five wait states of a vector instruction writing it; the
# compiler pads that hazard in front of its own loads, but the staging loads are inline assembly
# (a reloaded resource word or offset read too early fetched the previous tile's rows).  (About 1 KB of scratch per
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
        m = re.search(r"(ScratchSize \[bytes/lane\]|SGPRs Spill|VGPRs Spill): (\d+)", line)
        if m and int(m.group(2)) > 0 and name and "gemm_bf16" in name:
            bad.append((name, m.group(1), int(m.group(2))))
    if bad:
        raise RuntimeError(f"{src}: kernels spill registers: {bad}")
    return obj


def _sgprs(text: str):
    """Scalar register numbers named in an operand string: s7, s[4:7]."""
    regs = set()
    for a, b in re.findall(r"\bs\[(\d+):(\d+)\]", text):
        regs.update(range(int(a), int(b) + 1))
    regs.update(int(n) for n in re.findall(r"\bs(\d+)\b", text))
    return regs


def lint_staging_hazards(src: str = "gemm_bf16.hip") -> None:
    """The direct-to-LDS staging loads are inline assembly, so the compiler's hazard recogniser does
    not see them.  One hazard matters: a vector-memory instruction must not read a scalar register
    within five wait states of a VECTOR instruction writing it (v_readfirstlane of a uniform value
    kept in vector registers, v_readlane of a spilled scalar).  This reads the generated ISA and
    refuses the build if a staging load (or a global load with a scalar base, the form of the
    row-offset loads) reads such a register too early."""
    res = subprocess.run(["hipcc", *FLAGS, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", "-"],
                         stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc -S failed on {src}")
    window = []   # (wait states this instruction provides, scalar registers a vector instruction wrote)
    bad = []
    for ln, line in enumerate(res.stdout.splitlines(), 1):
        t = line.strip()
        if not t or t[0] in ";." or t.endswith(":") or t.startswith(("//", "#")):
            if t.endswith(":"):
                window = []          # a label: the predecessors are unknown, start over
            continue
        op = t.split()[0]
        if (op.startswith("buffer_load") and t.endswith("lds")) or (op.startswith("global_load") and "s[" in t):
            need, used = 5, _sgprs(t.split(None, 1)[1])
            for states, written in reversed(window):
                if need <= 0:
                    break
                if written & used:
                    bad.append((ln, t, sorted(written & used)))
                    break
                need -= states
        written = set()
        if op.startswith(("v_readfirstlane", "v_readlane")) or (op.startswith("v_cmp") and "_e64" in op):
            written = _sgprs(t.split(None, 1)[1].split(",")[0])
        states = 1
        if op == "s_nop":
            states = int(t.split()[1]) + 1
        window.append((states, written))
        del window[:-8]
    if bad:
        raise RuntimeError(f"{src}: staging loads read scalar registers too soon after a vector write: {bad[:5]}")


def build_library(jobs: int = 7) -> str:
    """Compile every translation unit and link the shared library.  Always rebuilds."""
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        lint = ex.submit(lint_staging_hazards)
        objs = list(ex.map(_compile, SOURCES))
        lint.result()
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
