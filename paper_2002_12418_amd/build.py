"""Builds libmnnconv.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2002_12418_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG), "include")
OBJ_DIR = os.path.join(PKG, "_build")
LIB_PATH = os.path.join(PKG, "libmnnconv.so")

SOURCES = ["api.cpp", "transforms.hip", "transforms_rect.hip", "gemm.hip", "weight_layout.hip", "fill.hip", "static_scratch.hip", "wino_fused.hip", "gemm_bf16.hip", "strassen.hip", "microbench.hip"]

# -packed-fp32-ops is switched off: hand-checked scalar fp32 code only.
COMMON = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-I", INCLUDE, "-I", CSRC,
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
          "-Wno-unknown-warning-option"]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP library cannot be built")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    extra = os.environ.get("MNNCONV_EXTRA_HIPCC_FLAGS", "").split()      # e.g. -DNAME=value for tuning experiments
    cmd = [_hipcc(), "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + COMMON + extra
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build_library(verbose: bool = True) -> str:
    """Compile every source for gfx950 and link paper_2002_12418_amd/libmnnconv.so."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    wanted = {os.path.splitext(src)[0] + ".o" for src in SOURCES}
    for stale in os.listdir(OBJ_DIR):                      # objects of sources that were renamed or removed
        if stale.endswith(".o") and stale not in wanted:
            os.remove(os.path.join(OBJ_DIR, stale))
    with ThreadPoolExecutor(max_workers=min(6, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB_PATH + ".tmp"
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    os.replace(tmp, LIB_PATH)
    if verbose:
        print(f"built {LIB_PATH} ({os.path.getsize(LIB_PATH) // 1024} KiB)")
    return LIB_PATH


if __name__ == "__main__":
    build_library()
