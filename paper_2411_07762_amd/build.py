"""Builds libaser.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2411_07762_amd.build

hipcc cross-compiles without a GPU.  Packed-fp32 VALU ops are switched off for all device code.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libaser.so")
CLIENT = os.path.join(PKG, "aser_abi_client")            # tests/native/abi_client.cpp: a caller without Python or PyTorch
CLIENT_SRC = os.path.join(ROOT, "tests", "native", "abi_client.cpp")
OBJDIR = os.path.join(PKG, "_build")

SOURCES = ["api.hip", "gemm_tn.hip", "bandwidth.hip", "smooth.hip", "dense_small.hip", "chol_block.hip", "eig_sym.hip", "whiten.hip", "reconstruct.hip", "spectrum.hip", "evaluate.hip", "forward.hip", "probe.hip", "layers.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-I", INCLUDE, "-I", CSRC]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> str:
    obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    return obj


def build_library(verbose: bool = True) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp"
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB, file=sys.stderr)
    if os.path.exists(CLIENT_SRC):
        cmd = [_hipcc(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", INCLUDE, CLIENT_SRC, "-o", CLIENT + ".tmp",
               "-L", PKG, "-laser", "-Wl,-rpath,$ORIGIN"]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("building the native client failed:\n%s\n%s" % (res.stdout, res.stderr))
        os.replace(CLIENT + ".tmp", CLIENT)
        if verbose:
            print("built", CLIENT, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build_library()
