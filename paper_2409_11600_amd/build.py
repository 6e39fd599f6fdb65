"""Builds libnsk.so (the HIP kernels + C ABI) for gfx950 with hipcc, in-tree next to this file."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libnsk.so")
OBJ = os.path.join(HERE, "_build")

SOURCES = ["nsk_api.hip", "conv_igemm.hip", "conv_igemm_big.hip", "conv_pw.hip", "conv_pw_narrow16.hip", "conv_pw_narrow32.hip", "conv_halo64.hip", "conv_fs64_s2.hip", "conv_halo_wide.hip", "conv_halo64_f32.hip", "conv_wgrad.hip", "conv_depthwise.hip", "conv_tiny.hip", "conv_wgrad_halo64.hip", "conv_wgrad_wide.hip", "conv_stem.hip", "conv_stem_halo.hip", "layout.hip", "bn.hip", "pool.hip", "tail.hip", "recurrent.hip", "pool_mem.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", INCLUDE, "-I", CSRC]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 target feature and says so on every file
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    """Compiles every source (always: this is the does-it-build check) and links libnsk.so."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
