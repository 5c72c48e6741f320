"""Builds libgspn.so (hand-written HIP, gfx950) in-tree with hipcc.

    python -m paper_2512_07884_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libgspn.so")
SOURCES = ["gspn_api.hip", "gspn_dispatch.hip", "gspn_generic.hip", "gspn_unfused.hip", "gspn_fwd_tile.hip", "gspn_fwd_tile_f32_global.hip", "gspn_fwd_tile_f32_local.hip", "gspn_fwd_tile_bf16_global.hip", "gspn_fwd_tile_bf16_local.hip", "gspn_fwd_stream.hip", "gspn_fwd_stream_f32.hip", "gspn_fwd_stream_bf16.hip", "gspn_fwd_stream_staged.hip", "gspn_fwd_plane.hip", "gspn_fwd_pair.hip", "gspn_bwd_tile.hip", "gspn_bwd_plane.hip", "gspn_bwd_twopass.hip", "gspn_bwd_twopass_f32.hip", "gspn_bwd_twopass_bf16.hip", "gspn_bwd_twopass_f32_local.hip", "gspn_bwd_twopass_bf16_local.hip", "gspn_proxy.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fno-gpu-rdc", "-Wall", "-Wno-unused-function"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + r.stdout + "\n" + err)
    return err


def build(verbose: bool = True) -> str:
    """Compiles every source to an object (in parallel, at most 8 at a time) and links the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    import shutil
    tmp = os.path.join(PKG, "_build")          # objects only; removed again below
    os.makedirs(tmp, exist_ok=True)
    try:
        jobs = []
        for src in SOURCES:
            obj = os.path.join(tmp, src.replace(".hip", ".o"))
            jobs.append(([HIPCC] + [f for f in FLAGS if f != "-shared"] + ["-c", os.path.join(CSRC, src), "-o", obj], obj))
        if verbose:
            for cmd, _ in jobs:
                print(" ".join(cmd), flush=True)
        with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
            errs = list(pool.map(_run, [cmd for cmd, _ in jobs]))
        link = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950"] + [obj for _, obj in jobs] + ["-o", LIB]
        if verbose:
            print(" ".join(link), flush=True)
        errs.append(_run(link))
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    if verbose and any(e.strip() for e in errs):
        print("\n".join(e for e in errs if e.strip()), file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build())
