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
SOURCES = ["gspn_api.hip", "gspn_dispatch.hip", "gspn_generic.hip", "gspn_unfused.hip", "gspn_fwd_tile.hip", "gspn_fwd_tile_f32_global.hip", "gspn_fwd_tile_f32_local.hip", "gspn_fwd_tile_bf16_global.hip", "gspn_fwd_tile_bf16_local.hip", "gspn_fwd_tile_f16_global.hip", "gspn_fwd_tile_f16_local.hip", "gspn_fwd_stream.hip", "gspn_fwd_stream_f32.hip", "gspn_fwd_stream_bf16.hip", "gspn_fwd_stream_f16.hip", "gspn_fwd_stream_staged.hip", "gspn_fwd_stream_staged_bf16.hip", "gspn_fwd_stream_staged_f16.hip", "gspn_fwd_stream_staged_bf16_local.hip", "gspn_fwd_stream_staged_f16_local.hip", "gspn_fwd_stream_staged_bf16_logits.hip", "gspn_fwd_stream_staged_f16_logits.hip", "gspn_fwd_stream_big.hip", "gspn_fwd_stream_big_global.hip", "gspn_fwd_stream_big_local.hip", "gspn_fwd_stream_big_logits.hip", "gspn_fwd_plane.hip", "gspn_fwd_pair.hip", "gspn_fwd_pair_bf16.hip", "gspn_fwd_pair_f16.hip", "gspn_fwd_chunk.hip", "gspn_bwd_tile.hip", "gspn_bwd_plane.hip", "gspn_bwd_twopass.hip", "gspn_bwd_twopass_f32.hip", "gspn_bwd_twopass_bf16.hip", "gspn_bwd_twopass_f32_local.hip", "gspn_bwd_twopass_bf16_local.hip", "gspn_bwd_twopass_f16.hip", "gspn_bwd_twopass_f16_local.hip", "gspn_proxy.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fno-gpu-rdc", "-Wall", "-Wno-unused-function"]
# The compiler reports every kernel's register and scratch use (-Rpass-analysis=kernel-resource-usage); the build fails
# when a kernel spills vector registers, because a spilled hot loop is slow and was once seen to return wrong values.
# Exceptions, by mangled-name fragment -> most registers it may spill, each with its reason:
SPILL_ALLOWED = {
    # reverse sweep of the staged stream kernel: one 16-byte value parked around the first request of y, before the
    # chunk loop (nothing inside it); parity-tested on 256x256 .. 512x512 maps
    "fwd_stream_staged_kernelItLi4ELi4ELb1ELb1": 16, "fwd_stream_staged_kernelItLi8ELi4ELb1ELb1": 16,
    "fwd_stream_staged_kernelItLi16ELi2ELb1ELb1": 16,
    "fwd_stream_staged_kernelINS_5f16_tELi4ELi4ELb1ELb1": 16, "fwd_stream_staged_kernelINS_5f16_tELi8ELi4ELb1ELb1": 16,
    "fwd_stream_staged_kernelINS_5f16_tELi16ELi2ELb1ELb1": 16,
    # ... with two channels of a group per workgroup: five 16-byte values parked while a chunk is turned into row order,
    # between the 64-step loops (none inside them); parity-tested on the same maps, train512 backward 2.24 -> 2.15 ms
    "fwd_stream_staged2_kernelItLi4ELi4ELb1ELb1": 67, "fwd_stream_staged2_kernelItLi8ELi4ELb1ELb1": 67,
    "fwd_stream_staged2_kernelItLi16ELi2ELb1ELb1": 67,
    "fwd_stream_staged2_kernelINS_5f16_tELi4ELi4ELb1ELb1": 67, "fwd_stream_staged2_kernelINS_5f16_tELi8ELi4ELb1ELb1": 67,
    "fwd_stream_staged2_kernelINS_5f16_tELi16ELi2ELb1ELb1": 67,
    # (65 values in the global scan's reverse sweep in bf16, 67 in fp16 and in GSPN-local's)
    # ... with the weights as logits (a softmax per scan step beside the chunk registers): values parked in scratch memory
    # around the step loops of the forward call with h_save (36) and of the reverse sweep (99 with one channel per
    # workgroup, 84 with two); these calls ran the general stream kernel before (long512 with logits 1.55 -> 1.13 ms);
    # parity-tested on 256- and 512-row maps in bf16 and fp16
    "fwd_stream_staged2_kernelItLi4ELi4ELb1ELb1ELb1ELb1": 84, "fwd_stream_staged_kernelItLi4ELi4ELb1ELb1ELb1ELb1": 99, "fwd_stream_staged_kernelItLi4ELi4ELb1ELb0ELb1ELb1": 36,
    "fwd_stream_staged2_kernelItLi8ELi4ELb1ELb1ELb1ELb1": 84, "fwd_stream_staged_kernelItLi8ELi4ELb1ELb1ELb1ELb1": 99, "fwd_stream_staged_kernelItLi8ELi4ELb1ELb0ELb1ELb1": 36,
    "fwd_stream_staged2_kernelItLi16ELi2ELb1ELb1ELb1ELb1": 84, "fwd_stream_staged_kernelItLi16ELi2ELb1ELb1ELb1ELb1": 99, "fwd_stream_staged_kernelItLi16ELi2ELb1ELb0ELb1ELb1": 36,
    "fwd_stream_staged2_kernelINS_5f16_tELi4ELi4ELb1ELb1ELb1ELb1": 84, "fwd_stream_staged_kernelINS_5f16_tELi4ELi4ELb1ELb1ELb1ELb1": 99, "fwd_stream_staged_kernelINS_5f16_tELi4ELi4ELb1ELb0ELb1ELb1": 36,
    "fwd_stream_staged2_kernelINS_5f16_tELi8ELi4ELb1ELb1ELb1ELb1": 84, "fwd_stream_staged_kernelINS_5f16_tELi8ELi4ELb1ELb1ELb1ELb1": 99, "fwd_stream_staged_kernelINS_5f16_tELi8ELi4ELb1ELb0ELb1ELb1": 36,
    "fwd_stream_staged2_kernelINS_5f16_tELi16ELi2ELb1ELb1ELb1ELb1": 84, "fwd_stream_staged_kernelINS_5f16_tELi16ELi2ELb1ELb1ELb1ELb1": 99, "fwd_stream_staged_kernelINS_5f16_tELi16ELi2ELb1ELb0ELb1ELb1": 36,
    # sixteen-wave horizontal kernel for maps of up to 1024 rows (128 registers per lane), with h_save or as the reverse
    # sweep: loop-invariant addresses parked before the chunk loop and read back once per chunk of 16 / 32 scan steps,
    # between the step loops (no scratch access inside them)
    "stream_big_horizontal_kernelItLi32ELb0ELb1": 7, "stream_big_horizontal_kernelItLi32ELb1ELb1": 5,
    "stream_big_horizontal_kernelIfLi16ELb1ELb1": 5,
    "stream_big_horizontal_kernelINS_5f16_tELi32ELb0ELb1": 5, "stream_big_horizontal_kernelINS_5f16_tELi32ELb1ELb1": 1,
    # ... with logits normalised on the way in (a softmax per position beside the 128 registers): up to 111 values in
    # scratch memory in the forward call with h_save, 25 in the reverse sweep; these calls ran the generic kernel before
    # (scale1024 with kchunk 128: 46.5 ms there, 4.1 ms on these kernels; with logits 4.3 ms); parity-tested on maps of
    # 576 to 1024 rows in the three storage types
    "stream_big_horizontal_kernelItLi32ELb0ELb1ELb1ELb1": 111, "stream_big_horizontal_kernelINS_5f16_tELi32ELb0ELb1ELb1ELb1": 111,
    "stream_big_horizontal_kernelItLi32ELb1ELb1ELb1ELb1": 25, "stream_big_horizontal_kernelINS_5f16_tELi32ELb1ELb1ELb1ELb1": 25,
    "stream_big_horizontal_kernelIfLi16ELb1ELb1ELb1ELb1": 5,
    # two-channel kernel, forward with h_save on raw logits: values parked in the accumulation registers (no scratch
    # memory: the kernel's ScratchSize is 0), none in the loop over the bands of the vertical phases, 4 to 16 moves per
    # step of the horizontal ones beside six exponentials; parity-tested at full size, train128 forward on logits
    # 0.569 ms on the one-channel tile kernel -> 0.426 ms
    "fwd_pair_kernelItLb1ELb0ELb1ELb1": 144,
    # the same in fp16 storage, and its GSPN-local forward with h_save (96 values, none in the band loop either; the
    # hardware conversions hold a few registers more than the shifts of bf16): parity-tested at full size
    "fwd_pair_kernelINS_5f16_tELb1ELb0ELb1ELb1": 144, "fwd_pair_kernelINS_5f16_tELb1ELb0ELb1ELb0": 96,
    # fp32 maps with rows of 112 bytes on workgroups of more than four waves, without h_save: off every benchmark shape
    # (the plane kernel takes 28x28, the four-wave instantiation 56x56); kept because the shapes must run somewhere
    "fwd_tile_kernelIfLi2ELi1ELi28ELb0ELi8ELb0ELi8ELb0ELb0ELb0": 259, "fwd_tile_kernelIfLi2ELi1ELi28ELb0ELi8ELb0ELi8ELb1ELb0ELb0": 47,
}


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("is not a recognized feature for this target", "[-Rpass-analysis=kernel-resource-usage]")
    err = "\n".join(l for l in r.stderr.splitlines() if not any(n in l for n in noise))
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + r.stdout + "\n" + err)
    _check_spills(r.stderr, cmd[-3] if len(cmd) > 3 else "")
    # the remarks quote a source line and a caret after each entry: drop what is left of them
    err = "\n".join(l for l in err.splitlines() if "__global__" not in l and l.strip() not in ("^", "|", "") and " | " not in l
                    and not l.startswith("In file included from"))
    return err


def _check_spills(stderr: str, what: str):
    """Raises when a kernel spills vector registers beyond what SPILL_ALLOWED grants it."""
    import re
    name = None
    bad = []
    for line in stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"VGPRs Spill: (\d+)", line)
        if m and name is not None:
            n = int(m.group(1))
            allowed = max([v for k, v in SPILL_ALLOWED.items() if k in name] or [0])
            if n > allowed:
                bad.append(f"{name}: {n} vector registers spilled (allowed: {allowed})")
    if bad:
        raise RuntimeError("register spills in " + what + ":\n  " + "\n  ".join(bad))


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
            jobs.append(([HIPCC] + [f for f in FLAGS if f != "-shared"] + ["-Rpass-analysis=kernel-resource-usage"]
                         + ["-c", os.path.join(CSRC, src), "-o", obj], obj))
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
