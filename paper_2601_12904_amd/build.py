"""Builds libfusionrag.so (gfx950 only) in-tree with hipcc.  `python -m paper_2601_12904_amd.build`."""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libfusionrag.so")

SOURCES = ["fr_api.cpp", "k_rope.hip", "k_scatter.hip", "k_score_simt.hip", "k_score_mfma.hip", "k_score_raw.hip", "k_select.hip", "k_select_large.hip", "fr_select_static.hip", "k_deviation.hip", "k_decode.hip",
           "k_attn_simt.hip", "k_attn_mfma.hip", "k_gemm.hip"]

FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # keep packed fp32 ops out of the code
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    noise = "'-packed-fp32-ops' is not a recognized feature"
    warn = "\n".join(l for l in r.stderr.splitlines() if l.strip() and noise not in l)
    return warn


def build(verbose: bool = False, extra_flags=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        warns = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    if verbose:
        for s, w in zip(SOURCES, warns):
            if w:
                print(f"[{s}]\n{w}", file=sys.stderr)
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
