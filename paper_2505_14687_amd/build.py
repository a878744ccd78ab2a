"""Compile libgrat.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libgrat.so")
# attn_mfma_*.hip: the instantiations of the MFMA kernel template (attn_mfma.h), one slice per
# element type and head_dim, so that the slow part of the build runs side by side
SOURCES = ["grat_api.hip", "block_lists.hip", "attn_f32.hip", "mfma_probe.hip", "attn_mfma.hip",
           "attn_mfma_bf16_d128.hip", "attn_mfma_bf16_d64.hip", "attn_mfma_f16_d128.hip", "attn_mfma_f16_d64.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # the packed-fp32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    # (the direct-to-LDS loads name m0 as clobbered on purpose)
    "-Wno-inline-asm",
]


def hipcc_path() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libgrat needs the ROCm toolchain to build")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    return res.stderr


def build_library(verbose: bool = False, extra_flags=(), jobs: int = 8) -> str:
    """Always recompiles every source (objects go to a scratch directory); returns the library path."""
    hipcc = hipcc_path()
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="libgrat_build_") as tmp:
        objs = [os.path.join(tmp, os.path.splitext(s)[0] + ".o") for s in SOURCES]

        def compile_one(pair):
            src, obj = pair
            return _run([hipcc, *HIPCC_FLAGS, *extra_flags, *inc, "-c", os.path.join(CSRC, src), "-o", obj], verbose)

        with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as ex:
            warnings = list(ex.map(compile_one, zip(SOURCES, objs)))
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH], verbose)
    if verbose:
        for w in warnings:
            w = "\n".join(l for l in w.splitlines() if "packed-fp32-ops" not in l)
            if w.strip():
                print(w)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
