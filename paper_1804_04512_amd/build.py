"""Builds libdll_conv.so (gfx950 only) in-tree with hipcc.

Usage: python -m paper_1804_04512_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdll_conv.so")
SOURCES = ["conv_engine.hip", "conv_fewout.hip", "conv_fwd_fewch.hip", "conv_fft.hip", "conv_wino.hip", "conv_wino_stream.hip", "conv_wgrad.hip", "conv_wgrad_wino.hip", "conv_wgrad_fewch.hip", "gemm.hip", "gemm_small.hip", "rbm.hip", "api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 VALU forms are switched off on purpose: the compiler then emits no v_pk_*_f32 instructions
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str, folder: str = CSRC) -> str:
    obj = os.path.join(folder, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(folder, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build() -> str:
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    return LIB


def build_program(src_path: str, out_path: str) -> str:
    """Compiles one stand-alone HIP program (same flags as the library)."""
    folder, src = os.path.split(src_path)
    obj = _compile(src, folder)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-o", out_path, obj], check=True)
    os.remove(obj)
    return out_path


if __name__ == "__main__":
    print(build())
