"""Builds libat_grpo.so (HIP, gfx950) in-tree with hipcc.  Run: python -m paper_2510_11062_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libat_grpo.so")
CLIENT = os.path.join(PKG, "abi_client")
PROBE = os.path.join(PKG, "gemm_probe")
SOURCES = ["api.hip", "group_advantage.hip", "token_kernels.hip", "head_kernels.hip", "optimizer.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.run(cmd, check=True)
    return obj


def build_client(verbose: bool = True) -> str:
    """A plain C99 caller of the library (gcc, the HIP C API): proof that the header is C and that the
    struct layout a C compiler produces is the one the library reads."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.environ.get("CC", "gcc"), "-std=c99", "-O1", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"),
           os.path.join(CSRC, "abi_client.c"), "-o", CLIENT, "-L", PKG, "-lat_grpo",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", CLIENT)
    return CLIENT


def build_probe(verbose: bool = True) -> str:
    """The tile loops as plain GEMMs (measurement aid, see csrc/gemm_probe.hip and bench_gemm.py)."""
    cmd = [HIPCC, *[f for f in FLAGS if f != "-fPIC"], os.path.join(CSRC, "gemm_probe.hip"), "-o", PROBE]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", PROBE)
    return PROBE


def build(verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    build_client(verbose)
    build_probe(verbose)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
