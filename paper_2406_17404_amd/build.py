"""Builds libtrjacobi.so (HIP kernels + C-ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtrjacobi.so")
SOURCES = ["api.hip", "tree_kernels.hip", "f32_kernels.hip", "gemm_bf16.hip", "attn_bf16.hip",
           "decode_loop.hip", "loop_host.cpp"]
# -packed-fp32-ops is a DEVICE code generation feature: with it hipcc emits no v_pk_*_f32
# from float code (checked on the device assembly of a float2 kernel: one v_pk_fma_f32
# without the flag, none with it).  The host pass of the same command does not know the
# feature and prints "not a recognized feature for this target": harmless, and left
# visible.
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    if src.endswith(".cpp"):   # host-only C++: no device pass, no device flags
        cmd = ["g++", "-O2", "-fPIC", "-std=c++17", "-Wall", "-c", os.path.join(CSRC, src), "-o", obj]
    else:
        cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"compiler failed on {src}:\n{r.stderr}")
    if r.stderr.strip():
        print(r.stderr, file=sys.stderr)
    return obj


def build_host_logic_sanitized(out_path: str) -> str:
    """The GPU-free part of the library (the decoding loop's host logic) as a shared library
    of its own under AddressSanitizer and UndefinedBehaviorSanitizer; for tests."""
    cmd = ["g++", "-O1", "-g", "-fPIC", "-shared", "-std=c++17", "-Wall", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", os.path.join(CSRC, "loop_host.cpp"),
           "-o", out_path]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("sanitized host build failed:\n" + r.stderr)
    return out_path


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
