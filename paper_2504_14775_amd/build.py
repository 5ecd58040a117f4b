"""Builds libgllm_stage.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2504_14775_amd.build
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgllm_stage.so")
BUILD_DIR = os.path.join(HERE, "_build")
SOURCES = ["gllm_stage.hip", "kernels_gemm.hip", "kernels_attn.hip", "kernels_misc.hip", "kernels_peak.hip",
           "gllm_head.hip", "gllm_sched.cpp", "gllm_kv.cpp"]   # the last two are host code only (scheduler, KV page pool)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> str:
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + ".o")
    flags = FLAGS if src.endswith(".hip") else ["-O2", "-std=c++17", "-fPIC", "-Wall"]
    cmd = [hipcc(), *flags, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print("built", LIB)
    return LIB


HOST_SOURCES = ["gllm_sched.cpp", "gllm_kv.cpp"]
HOST_SAN_LIB = os.path.join(BUILD_DIR, "libgllm_host_san.so")


def build_host_sanitized() -> str:
    """The host-only sources (scheduler, KV page pool) as a library of their own with AddressSanitizer and
    UndefinedBehaviorSanitizer (g++, CPU only); a process that loads it must have the ASan runtime preloaded."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    cxx = shutil.which("g++") or "g++"
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fPIC", "-shared", "-Wall", "-o", HOST_SAN_LIB,
           *[os.path.join(CSRC, f) for f in HOST_SOURCES]]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"sanitizer build failed:\n{r.stdout}\n{r.stderr}")
    return HOST_SAN_LIB


def sanitizer_runtime() -> str:
    cxx = shutil.which("g++") or "g++"
    return subprocess.run([cxx, "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()


if __name__ == "__main__":
    build()
