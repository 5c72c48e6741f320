#!/usr/bin/env python3
"""Benchmark of the fused 4-direction GSPN scan on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--kchunk K] [--logits] [--storage f32|bf16|f16] [--throughput-table] [--all]

A step is one pass of the whole hot path over one batch of synthetic input:
one ``gspn_scan_fwd`` call covering all four directions (inference workloads),
or ``gspn_scan_fwd`` (saving h) + ``gspn_scan_bwd`` (training workloads).
Inputs are resident in HBM before the timed region; buffer sets are rotated so
that consecutive steps do not find their inputs in the 256 MB last-level cache.
Prints ONE JSON line (see the keys below); ``--all`` additionally writes a table
for every workload to <out>/bench_all.json (see --out).  ``--kchunk K`` times the
GSPN-local calls (propagation confined to stretches of K lines) on the same workload; ``--logits``
the calls that take the weights as raw logits and normalise them inside.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
DEFAULT_WORKLOAD = "diff128"   # 128x128 diffusion-latent shape: first of the two target shapes
TRAINING = ("train28_gc", "train28_g4", "train56", "train128", "train512", "occ128_train")


def device_inputs(cfg, seed: int, logits: bool = False):
    """Synthetic inputs with the distributions of workloads.make_slice, drawn on the device."""
    import torch
    td = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[cfg.dtype]
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    B, C, H, W, G = cfg.B, cfg.C, cfg.H, cfg.W, cfg.G
    x = torch.randn((B, C, H, W), generator=g, device="cuda").to(td)
    w = torch.empty((4, B, G, 3, H, W), dtype=td, device="cuda")
    lam = torch.empty((4, B, C, H, W), dtype=td, device="cuda")
    u = torch.empty((4, B, C, H, W), dtype=td, device="cuda")
    for d in range(4):
        z = torch.randn((B, G, 3, H, W), generator=g, device="cuda") * cfg.logit_scale
        if d < 2:
            z[:, :, 0, :, 0] = float("-inf"); z[:, :, 2, :, -1] = float("-inf")
        else:
            z[:, :, 0, 0, :] = float("-inf"); z[:, :, 2, -1, :] = float("-inf")
        w[d] = z.nan_to_num(neginf=0.0).to(td) if logits else torch.softmax(z.double(), dim=2).to(td)
        lam[d] = torch.rand((B, C, H, W), generator=g, device="cuda").to(td)
        u[d] = torch.rand((B, C, H, W), generator=g, device="cuda").to(td)
        del z
    gy = torch.randn((B, C, H, W), generator=g, device="cuda").to(td)
    return {"x": x, "w": w, "lam": lam, "u": u, "gy": gy}


def make_sets(cfg, training: bool, min_total_bytes: float = 1.0e9, max_sets: int = 4, logits: bool = False):
    import torch
    foot = cfg.fwd_algorithmic_bytes(save_h=training) + (cfg.bwd_algorithmic_bytes() if training else 0)
    nsets = int(min(max_sets, max(1, math.ceil(min_total_bytes / foot))))
    sets = []
    for i in range(nsets):
        s = device_inputs(cfg, 1000 + i, logits)
        s["y"] = torch.empty_like(s["x"])
        if training:
            s["hs"] = torch.empty_like(s["lam"])
            s["gx"] = torch.empty_like(s["x"])
            s["gw"] = torch.empty_like(s["w"])
            s["glam"] = torch.empty_like(s["lam"])
            s["gu"] = torch.empty_like(s["lam"])
        sets.append(s)
    return sets


def run_workload(cfg, steps: int, warmup: int, kchunk: int = 0, logits: bool = False, transposed: bool = False):
    """Times `steps` steps; returns dict with wall ms/step and per-kernel event times."""
    import torch
    import paper_2512_07884_amd as G
    training = cfg.name in TRAINING
    sets = make_sets(cfg, training, logits=logits)
    stream = torch.cuda.current_stream()
    big = 1 << 14
    if transposed:      # x in both layouts; the parameter slots of directions 2, 3 are read as [.., W, H] (random data)
        for s_ in sets:
            s_["xt"] = s_["x"].transpose(-1, -2).contiguous()

    def fwd(s):
        if transposed:
            G.gspn_scan_fwd_transposed(s["x"], s["xt"], s["w"], s["lam"], s["u"], s["y"], G=cfg.G, dir_mask=cfg.dir_mask)
        elif logits:
            G.gspn_scan_fwd_logits(s["x"], s["w"], s["lam"], s["u"], s["y"], s.get("hs"), kchunk=kchunk or big, G=cfg.G,
                                   dir_mask=cfg.dir_mask)
        elif kchunk:
            G.gspn_scan_fwd_local(s["x"], s["w"], s["lam"], s["u"], s["y"], s.get("hs"), kchunk=kchunk, G=cfg.G,
                                  dir_mask=cfg.dir_mask)
        else:
            G.gspn_scan_fwd(s["x"], s["w"], s["lam"], s["u"], s["y"], s.get("hs"), G=cfg.G, dir_mask=cfg.dir_mask)

    def bwd(s):
        if logits:
            G.gspn_scan_bwd_logits(s["gy"], s["x"], s["w"], s["lam"], s["u"], s["hs"], s["gx"], s["gw"], s["glam"],
                                   s["gu"], kchunk=kchunk or big, G=cfg.G, dir_mask=cfg.dir_mask)
        elif kchunk:
            G.gspn_scan_bwd_local(s["gy"], s["x"], s["w"], s["lam"], s["u"], s["hs"], s["gx"], s["gw"], s["glam"],
                                  s["gu"], kchunk=kchunk, G=cfg.G, dir_mask=cfg.dir_mask)
        else:
            G.gspn_scan_bwd(s["gy"], s["x"], s["w"], s["lam"], s["u"], s["hs"], s["gx"], s["gw"], s["glam"],
                            s["gu"], G=cfg.G, dir_mask=cfg.dir_mask)

    for i in range(warmup):
        s = sets[i % len(sets)]
        fwd(s)
        if training:
            bwd(s)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        s = sets[i % len(sets)]
        ev[i][0].record(stream)
        fwd(s)
        ev[i][1].record(stream)
        if training:
            bwd(s)
            ev[i][2].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # warm figure, reported separately: the same step on ONE buffer set, back to back (inputs may sit in the
    # 256 MB last-level cache when they fit)
    wn = max(5, min(steps, 20))
    w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    w0.record(stream)
    for _ in range(wn):
        fwd(sets[0])
        if training:
            bwd(sets[0])
    w1.record(stream)
    torch.cuda.synchronize()
    warm_ms = w0.elapsed_time(w1) / wn
    fwd_ms = sorted(e[0].elapsed_time(e[1]) for e in ev)
    out = {"ms_per_step": (t1 - t0) * 1e3 / steps,
           "fwd_ms_avg": sum(fwd_ms) / steps, "fwd_ms_med": fwd_ms[steps // 2], "fwd_ms_min": fwd_ms[0],
           "n_sets": len(sets), "training": training, "warm_ms_per_step": warm_ms, "kchunk": kchunk, "logits": logits, "transposed": transposed}
    if training:
        bwd_ms = sorted(e[1].elapsed_time(e[2]) for e in ev)
        out.update({"bwd_ms_avg": sum(bwd_ms) / steps, "bwd_ms_med": bwd_ms[steps // 2], "bwd_ms_min": bwd_ms[0]})
    del sets
    torch.cuda.empty_cache()
    return out


def summarise(cfg, r):
    import paper_2512_07884_amd as G
    dt = {"f32": 0, "bf16": 1, "f16": 2}[cfg.dtype]
    training = r["training"]
    kchunk = r.get("kchunk", 0)
    big = 1 << 14                      # a stretch longer than any line: the global scan
    fplan, bplan = (G.gspn_fwd_logits_plan, G.gspn_bwd_logits_plan) if r.get("logits") else \
                   (G.gspn_fwd_local_plan, G.gspn_bwd_local_plan)
    if r.get("transposed"):
        fplan = lambda B, C, H, W, G_, k, mask, dt, flags, save: G.gspn_fwd_transposed_plan(B, C, H, W, G_, mask, dt, flags)
    fwd_bytes = cfg.fwd_algorithmic_bytes(save_h=training)
    d = {"workload": cfg.name, "B": cfg.B, "C": cfg.C, "H": cfg.H, "W": cfg.W, "G": cfg.G,
         "storage": cfg.dtype, "directions": cfg.n_dirs,
         "step": "fwd+bwd" if training else "fwd",
         "ms_per_step": r["ms_per_step"], "warm_single_set_ms_per_step": r["warm_ms_per_step"],
         "gpixel_ch_per_s": cfg.pixel_channels / (r["ms_per_step"] * 1e-3) / 1e9,
         "fwd_kernel": fplan(cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, kchunk or big, cfg.dir_mask, dt, 0, training),
         "fwd_ms_avg": r["fwd_ms_avg"], "fwd_ms_min": r["fwd_ms_min"],
         "fwd_algorithmic_bytes": fwd_bytes,
         "fwd_algorithmic_GBs": fwd_bytes / (r["fwd_ms_avg"] * 1e-3) / 1e9,
         "fwd_frac_of_hbm_peak": fwd_bytes / (r["fwd_ms_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
         "buffer_sets_rotated": r["n_sets"]}
    if kchunk:
        d["kchunk"] = kchunk
    if r.get("logits"):
        d["weights"] = "logits"
    if r.get("transposed"):
        # the fraction above stays on the algorithmic bytes of the scan; the second copy of x this layout reads is
        # counted in a figure of its own
        d["layout"] = "horizontal directions stored transposed (x read in both layouts: one more plane per pixel*channel)"
        with_xt = fwd_bytes + cfg.pixel_channels * cfg.elem_bytes
        d["fwd_bytes_incl_second_x"] = with_xt
        d["fwd_frac_of_hbm_peak_incl_second_x"] = with_xt / (r["fwd_ms_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS
    if training:
        bb = cfg.bwd_algorithmic_bytes()
        d.update({"bwd_kernel": bplan(cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, kchunk or big, cfg.dir_mask, dt, 0),
                  "bwd_ms_avg": r["bwd_ms_avg"], "bwd_ms_min": r["bwd_ms_min"],
                  "bwd_algorithmic_bytes": bb,
                  "bwd_algorithmic_GBs": bb / (r["bwd_ms_avg"] * 1e-3) / 1e9,
                  "bwd_frac_of_hbm_peak": bb / (r["bwd_ms_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS})
    return d


# ---------------------------------------------------------------- CPU baseline (the oracle, as it stands)
def _oracle_slice(args):
    name, b, g, training, kchunk, logits = args
    import numpy as np
    from oracle import gspn_oracle as O
    from paper_2512_07884_amd import workloads as WL
    cfg = WL.CONFIGS[name]
    s = WL.inputs_as_f64(WL.make_slice(cfg, b, g), cfg.dtype)
    t0 = time.perf_counter()
    a = (s["x"][None], s["w"][:, None, None], s["lam"][:, None], s["u"][:, None])
    if logits:      # the generated weights serve as logit values: same shapes, same cost
        y, h = O.scan_fwd_logits(*a, cfg.dir_mask, kchunk or None)
        if training:
            O.scan_bwd_logits(s["gy"][None], *a, h, cfg.dir_mask, kchunk or None)
    elif kchunk:
        y, h = O.scan_fwd_local(*a, kchunk, cfg.dir_mask)
        if training:
            O.scan_bwd_local(s["gy"][None], *a, h, kchunk, cfg.dir_mask)
    else:
        y, h = O.scan_fwd(*a, cfg.dir_mask)
        if training:
            O.scan_bwd(s["gy"][None], *a, h, cfg.dir_mask)
    return time.perf_counter() - t0, float(np.abs(y).sum())


def cpu_baseline(cfg, training: bool, budget_s: float = 12.0, kchunk: int = 0, logits: bool = False):
    """The fp64 NumPy oracle on (batch, group) slices of the same workload, one
    slice per worker process, timed wall-clock over the pool (input generation
    excluded from the single-slice probe, included in the pool's wall time is
    avoided by timing only the oracle calls and dividing by the worker count)."""
    import multiprocessing as mp
    cores = max(1, min(16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)))
    t_probe, _ = _oracle_slice((cfg.name, 0, 0, training, kchunk, logits))
    slice_pc = cfg.cpg * cfg.H * cfg.W
    total_slices = cfg.B * cfg.G
    n = int(max(cores, min(total_slices, (budget_s * cores) // max(t_probe, 1e-4))))
    n = min(n, total_slices)
    # a workload the oracle gets through in less than the budget is run several times over, so that the figure rests
    # on about budget_s seconds of CPU work
    passes = int(max(1, min(64, budget_s // max(n * t_probe, 1e-4))))
    jobs = [(cfg.name, (i // cfg.G) % cfg.B, i % cfg.G, training, kchunk, logits) for i in range(n)] * passes
    ctx = mp.get_context("fork")
    t0 = time.perf_counter()
    with ctx.Pool(min(cores, n)) as pool:
        res = pool.map(_oracle_slice, jobs, chunksize=1)
    wall = time.perf_counter() - t0
    busy = sum(r[0] for r in res)
    used = min(cores, n)
    # throughput of `used` workers running the oracle concurrently
    value = n * passes * slice_pc / (busy / used) / 1e9
    return {"value": value, "unit": "Gpixel*ch/s", "cores": used, "kind": "oracle",
            "sample": f"{n} of {total_slices} (batch, group) slices of {cfg.name}{f', {passes} times over' if passes > 1 else ''} "
                      f"({busy:.1f} s of CPU work), "
                      f"{'fwd+bwd' if training else 'fwd'}, fp64 NumPy, one slice per process; "
                      f"single-process rate {slice_pc / t_probe / 1e9:.4f} Gpixel*ch/s; pool wall {wall:.1f} s"}


def load_traffic(workload: str, dom: str):
    """Measured HBM bytes per launch of the dominant kernel (dom = "fwd" / "bwd"), from the
    rocprofv3 counter runs summarised in profiles/traffic.json (absent -> None)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(f"{dom}_hbm_bytes_per_launch")
    except (OSError, ValueError):
        return None


PROXY_SHAPES = (("classifier stage, C 96 -> 8", 64, 96, 8, 56, 56), ("classifier stage, back up 8 -> 96", 64, 8, 96, 56, 56),
                ("diffusion study, C 1152 -> 144", 2, 1152, 144, 128, 128), ("diffusion study, back up 144 -> 1152", 2, 144, 1152, 128, 128))


def proxy_table(steps: int = 50):
    """Compressive proxy projections (Sec. 4.2) on bf16 tensors: time per call and bytes moved (input read once,
    output written once, P negligible) against the HBM peak; buffer pairs rotated as in the scan benchmark."""
    import torch
    import paper_2512_07884_amd as G
    rows = []
    for name, B, K, M, H, W in PROXY_SHAPES:
        nbytes = 2 * B * (K + M) * H * W
        nsets = int(min(32, max(1, math.ceil(1.0e9 / nbytes))))     # >= 1 GB in rotation: past the last-level cache
        sets = [(torch.randn(B, K, H, W, device="cuda").to(torch.bfloat16),
                 (torch.randn(M, K, device="cuda") / K ** 0.5).to(torch.bfloat16),
                 torch.empty(B, M, H, W, device="cuda", dtype=torch.bfloat16)) for _ in range(nsets)]
        for i in range(5):
            G.gspn_proxy_project(*sets[i % nsets])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            G.gspn_proxy_project(*sets[i % nsets])
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        # its gradients: gin (reads gout, writes gin) and gP (reads gout and in; fp32 [M,K] through a [B,M,K] workspace)
        gin = torch.empty(B, K, H, W, device="cuda", dtype=torch.bfloat16)
        gP = torch.empty(M, K, device="cuda", dtype=torch.float32)
        part = torch.empty(B, M, K, device="cuda", dtype=torch.float32)
        bwd_ms = []
        for want in ((gin, None, None), (None, gP, part)):
            for i in range(5):
                x_, P_, o_ = sets[i % nsets]
                G.gspn_proxy_project_bwd(o_, x_, P_, *want)
            torch.cuda.synchronize()
            e0.record()
            for i in range(steps):
                x_, P_, o_ = sets[i % nsets]
                G.gspn_proxy_project_bwd(o_, x_, P_, *want)        # (the forward's output buffers serve as gout)
            e1.record()
            torch.cuda.synchronize()
            bwd_ms.append(e0.elapsed_time(e1) / steps)
        rows.append({"projection": name, "B": B, "K": K, "M": M, "H": H, "W": W, "kernel": G.gspn_proxy_plan(B, K, M, H, W, 1),
                     "ms": ms, "bytes": nbytes, "GBs": nbytes / (ms * 1e-3) / 1e9,
                     "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "TFLOPs": 2.0 * B * K * M * H * W / (ms * 1e-3) / 1e12,
                     "grad_input_ms": bwd_ms[0], "grad_input_GBs": nbytes / (bwd_ms[0] * 1e-3) / 1e9,
                     "grad_weight_ms": bwd_ms[1], "grad_weight_GBs": nbytes / (bwd_ms[1] * 1e-3) / 1e9})
        del sets, gin, gP, part
        torch.cuda.empty_cache()
    return rows


def unfused_table(steps: int = 3):
    """Fused against unfused on this hardware: the library's forward call beside the per-line-launch comparator
    (gspn_scan_fwd_unfused: one launch per line and direction, the state through global memory -- the structure of the
    first GSPN implementation, Sec. 3.3) on the shape of the paper's step-by-step study (Sec. 5.1: 1024x1024, B = 16,
    C = 8, where it reports 40x end to end on an A100) and on the two target shapes with few channels (Table 1 regime)."""
    import torch
    import paper_2512_07884_amd as G
    from paper_2512_07884_amd import workloads as WL
    rows = []
    for name, B, C, H, W, Gr, dtype in (("step-by-step study shape", 16, 8, 1024, 1024, 1, "f32"),
                                         ("step-by-step study shape, bf16", 16, 8, 1024, 1024, 1, "bf16"),
                                         ("512x512, 128 channels", 1, 128, 512, 512, 4, "bf16"),
                                         ("128x128, 2048 channels (diff128)", 2, 1024, 128, 128, 16, "bf16")):
        cfg = WL.ScanConfig("unfused_" + name, B, C, H, W, Gr, dtype, 15, 1.0, 7)
        s = device_inputs(cfg, 77)
        y = torch.empty_like(s["x"])
        ws = torch.empty(G.gspn_unfused_workspace_bytes(B, C, H, W), dtype=torch.uint8, device="cuda")
        dt = 1 if dtype == "bf16" else 0
        times = {}
        for kind in ("fused", "unfused"):
            def call():
                if kind == "fused":
                    G.gspn_scan_fwd(s["x"], s["w"], s["lam"], s["u"], y, None, G=Gr)
                else:
                    G.gspn_scan_fwd_unfused(s["x"], s["w"], s["lam"], s["u"], y, None, ws, G=Gr)
            call()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                call()
            torch.cuda.synchronize()
            times[kind] = (time.perf_counter() - t0) * 1e3 / steps
        rows.append({"shape": name, "B": B, "C": C, "H": H, "W": W, "G": Gr, "storage": dtype,
                     "fused_kernel": G.gspn_fwd_plan(B, C, H, W, Gr, 15, dt, 0, False),
                     "fused_ms": times["fused"], "unfused_ms": times["unfused"],
                     "launches_unfused": 2 * (H + W), "ratio": times["unfused"] / times["fused"]})
        del s, y, ws
        torch.cuda.empty_cache()
    return {"rows": rows, "paper_context": "GSPN-2 reports 40x (1024x1024, B=16, C=8), 36.8x and 151x over GSPN-1 on an "
                                            "NVIDIA A100 (Sec. 5.1): another machine and a tuned baseline; context, not a target"}


def chunk_axis_table(steps: int = 200, kchunk: int = 32):
    """GSPN-local on a call with few planes (Sec. 3.2, Sec. 4.1: the chunk index is part of the grid): the global scan
    beside the local one, whose stretches are work items of their own, on the low-occupancy shape of Table 1."""
    from paper_2512_07884_amd import workloads as WL
    rows = []
    for name in ("occ128", "occ128_train"):
        cfg = WL.CONFIGS[name]
        for dtype in ("f32", "bf16"):
            c = WL.shrink(cfg, dtype=dtype)
            g = summarise(c, run_workload(c, steps, 10))
            l = summarise(c, run_workload(c, steps, 10, kchunk))
            row = {"workload": f"{name}: B={c.B} C={c.C} H={c.H} W={c.W} G={c.G} {dtype}", "kchunk": kchunk,
                   "global_fwd_kernel": g["fwd_kernel"], "local_fwd_kernel": l["fwd_kernel"],
                   "global_fwd_ms": g["fwd_ms_avg"], "local_fwd_ms": l["fwd_ms_avg"],
                   "fwd_global_over_local": g["fwd_ms_avg"] / l["fwd_ms_avg"]}
            if "bwd_ms_avg" in g:
                row.update(global_bwd_ms=g["bwd_ms_avg"], local_bwd_ms=l["bwd_ms_avg"],
                           bwd_global_over_local=g["bwd_ms_avg"] / l["bwd_ms_avg"],
                           global_step_ms=g["ms_per_step"], local_step_ms=l["ms_per_step"])
            rows.append(row)
    return rows


# the eight shapes of the paper's global-memory throughput table (Table 1): (H = W, B, C).  The table gives neither the
# group count nor the storage type; eight channels per weight group (the ratio of the benchmark's classifier stage) and
# bf16 storage are taken here, and fp32 beside it
THROUGHPUT_TABLE_SHAPES = ((32, 32, 196), (64, 1, 768), (64, 1, 1152), (64, 1, 32), (128, 1, 32), (256, 1, 64), (256, 8, 64),
                           (512, 1, 128))


def throughput_table(steps: int = 100):
    """Forward scan on the shapes of Table 1: time per launch and the algorithmic bytes it moves per second.  (The paper's
    column is the memory throughput a profiler reports while its kernel runs; the figure here is the end-to-end one --
    compulsory bytes over launch time -- so shapes with fewer planes than the chip has compute units show their idle
    units in it.)"""
    from paper_2512_07884_amd import workloads as WL
    rows = []
    for hw, B, C in THROUGHPUT_TABLE_SHAPES:
        for dtype in ("bf16", "f32"):
            G_ = max(1, C // 8)
            while C % G_:
                G_ -= 1
            cfg = WL.ScanConfig(f"table1_{hw}_{B}_{C}", B, C, hw, hw, G_, dtype, 15, 1.0, 17)
            s = summarise(cfg, run_workload(cfg, steps, 10))
            rows.append({"shape": f"{hw}x{hw}, B={B}, C={C}, G={G_}, {dtype}", "planes": B * C, "kernel": s["fwd_kernel"],
                         "fwd_ms": s["fwd_ms_avg"], "algorithmic_bytes": s["fwd_algorithmic_bytes"],
                         "GBs": s["fwd_algorithmic_bytes"] / (s["fwd_ms_avg"] * 1e-3) / 1e9,
                         "frac_of_hbm_peak": s["fwd_algorithmic_bytes"] / (s["fwd_ms_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS})
    return rows


def copy_calibration(n_bytes: int = 1 << 30, reps: int = 5):
    """Plain copies of a known size: each must read and write exactly n_bytes, which
    fixes the unit in which the profiler's FETCH_SIZE / WRITE_SIZE counters report."""
    import torch
    src = torch.ones(n_bytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_calibration_bytes": n_bytes, "copies": reps}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--kchunk", type=int, default=0,
                    help="GSPN-local: confine propagation to stretches of this many lines (0: the global scan)")
    ap.add_argument("--storage", choices=("f32", "bf16", "f16"), default=None,
                    help="time the workload in this storage type instead of its own (fp16: the tile, stream and generic kernels)")
    ap.add_argument("--logits", action="store_true",
                    help="weights given as raw logits, normalised inside the call (gspn_scan_*_logits)")
    ap.add_argument("--transposed", action="store_true",
                    help="forward workloads: horizontal directions stored transposed (gspn_scan_fwd_transposed)")
    ap.add_argument("--proxy", action="store_true",
                    help="also time the compressive proxy projections (table under detail.proxy_projections)")
    ap.add_argument("--unfused", action="store_true",
                    help="also time the per-line-launch comparator against the fused forward (table under detail.fused_vs_unfused)")
    ap.add_argument("--chunk-axis", action="store_true",
                    help="also time GSPN-local against the global scan on the low-occupancy shape (detail.local_chunk_axis)")
    ap.add_argument("--throughput-table", action="store_true",
                    help="also time the forward scan on the eight shapes of the paper's throughput table (detail.throughput_table)")
    ap.add_argument("--all", action="store_true", help="also time every other workload (table in the --out folder)")
    ap.add_argument("--out", default="bench_out", help="folder for the --all table, relative to the repository root")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain 1 GiB device-to-device copies (known traffic, for scaling profiler counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build measures one GPU; the scan shards over (batch, group) with no "
              "exchange, and no multi-GPU figure is produced. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    if a.copy_calibration:
        copy_calibration()
        return
    from paper_2512_07884_amd import workloads as WL
    cfg = WL.CONFIGS[a.workload]
    other_storage = a.storage is not None and a.storage != cfg.dtype
    if other_storage:
        cfg = WL.shrink(cfg, dtype=a.storage)
    # the CPU legs fork worker processes: run them before this process touches the GPU
    if a.kchunk < 0:
        print("bench.py: --kchunk must be >= 0", file=sys.stderr)
        sys.exit(2)
    cpu = None if a.no_cpu else cpu_baseline(cfg, cfg.name in TRAINING, kchunk=a.kchunk, logits=a.logits)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if a.transposed and (cfg.name in TRAINING or a.kchunk or a.logits):
        print("bench.py: --transposed is a forward-only layout of the plain scan", file=sys.stderr)
        sys.exit(2)
    r = run_workload(cfg, a.steps, a.warmup, a.kchunk, a.logits, a.transposed)
    s = summarise(cfg, r)
    training = r["training"]
    dom = "bwd" if training else "fwd"          # dominant kernel of the step
    dom_bytes = s[f"{dom}_algorithmic_bytes"]
    dom_ms = s[f"{dom}_ms_avg"]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    line = {
        "metric": "GSPN 4-dir scan Gpixel*ch/s",
        "value": s["gpixel_ch_per_s"], "unit": "Gpixel*ch/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": s["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "storage_dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} C={cfg.C} H={cfg.H} W={cfg.W} G={cfg.G} "
                               f"{cfg.dtype} storage, {cfg.n_dirs} directions, {s['step']}"
                               + (f", GSPN-local kchunk={a.kchunk}" if a.kchunk else "")
                               + (", weights as logits" if a.logits else "")
                               + (", horizontal directions stored transposed" if a.transposed else ""),
                   "kernel": s[f"{dom}_kernel"], "buffer_sets_rotated": s["buffer_sets_rotated"]},
        "roofline": {"bound": "hbm", "kernel": f"gspn_scan_{dom}", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None if (a.kchunk or a.logits or a.transposed or other_storage) else load_traffic(cfg.name, dom),
                     "traffic_source": "stored: profiles/traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier "
                                       "run of this command, scaled by a 1 GiB copy), not measured in this run",
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms},
        "detail": s,
    }
    if cfg.name == DEFAULT_WORKLOAD and not (a.kchunk or a.logits or a.transposed or other_storage):
        # The metric names two shapes, 128x128 and 512x512, forward and backward: beside the forward-only headline on
        # the first, the same figures (algorithmic bytes per launch, mean launch time from events on the launch
        # stream, fraction of the HBM peak) for the forward on the second and for both shapes as training steps
        # (forward with h_save + backward)
        keys = ("workload", "step", "ms_per_step", "gpixel_ch_per_s", "fwd_kernel", "fwd_ms_avg", "fwd_algorithmic_bytes",
                "fwd_algorithmic_GBs", "fwd_frac_of_hbm_peak", "bwd_kernel", "bwd_ms_avg", "bwd_algorithmic_bytes",
                "bwd_algorithmic_GBs", "bwd_frac_of_hbm_peak")
        targets = [{k: s[k] for k in keys if k in s}]
        for name, div in (("long512", 4), ("train128", 4), ("train512", 8)):
            ct = WL.CONFIGS[name]
            t = summarise(ct, run_workload(ct, max(10, a.steps // div), min(a.warmup, 5)))
            targets.append({k: t[k] for k in keys if k in t})
        line["detail"]["target_shapes"] = targets
        line["detail"]["training_step_on_this_shape"] = targets[2]
    if cpu is not None:
        line["cpu_baseline"] = cpu
    if a.proxy:
        line["detail"]["proxy_projections"] = proxy_table()
    if a.unfused:
        line["detail"]["fused_vs_unfused"] = unfused_table()
    if a.chunk_axis:
        line["detail"]["local_chunk_axis"] = chunk_axis_table()
    if a.throughput_table:
        line["detail"]["throughput_table"] = throughput_table()
    if a.all:
        table = [s]
        for name, c in WL.CONFIGS.items():
            if name == cfg.name:
                continue
            k = max(20, a.steps // (8 if c.pixel_channels > 1e8 else 1))
            table.append(summarise(c, run_workload(c, k, a.warmup, a.kchunk, a.logits)))
            print(f"[bench] {name} done", file=sys.stderr, flush=True)
        os.makedirs(os.path.join(ROOT, a.out), exist_ok=True)
        with open(os.path.join(ROOT, a.out, "bench_all.json"), "w") as f:
            json.dump(table, f, indent=1)
        line["all_workloads"] = [{k: t[k] for k in t if k in (
            "workload", "step", "ms_per_step", "gpixel_ch_per_s", "fwd_ms_avg", "fwd_algorithmic_GBs",
            "fwd_frac_of_hbm_peak", "bwd_ms_avg", "bwd_algorithmic_GBs", "bwd_frac_of_hbm_peak", "fwd_kernel",
            "bwd_kernel")} for t in table]
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
