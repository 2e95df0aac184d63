"""Compile the HIP sources under csrc/ into libdpclip.so (gfx950 only), in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libdpclip.so")

SOURCES = ["dp_api.hip", "dp_small_kernels.hip", "dp_bias.hip", "dp_tn_bf16.hip", "dp_tn_bf16_dma.hip", "dp_tn_f32.hip", "dp_tn_f32_dma.hip", "dp_gram_bf16.hip", "dp_gram_cols.hip", "dp_conv_rows.hip", "dp_gram_bf16_dma.hip", "dp_gram_f32.hip", "dp_tn_f8_dma.hip", "dp_probes.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU ops are kept off for every HIP translation unit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = False, extra_flags=(), jobs: int = 8) -> str:
    """Compile every translation unit (in parallel, objects under _build/) and link them into libdpclip.so."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(PKG_DIR, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]

    def compile_one(name: str) -> str:
        obj = os.path.join(objdir, name + ".o")
        cmd = [hipcc_path(), *compile_flags, *extra_flags, "-c", os.path.join(CSRC, name), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {name}:\n" + res.stdout + res.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    tmp = LIB_PATH + ".tmp"
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
