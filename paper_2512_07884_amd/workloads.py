"""Seeded synthetic inputs for the GSPN scan, shaped like the paper's workloads.

This module holds no part of the method's arithmetic (no recurrence, no
merge): it only draws random tensors, normalises raw weight logits into the
row-stochastic tridiagonal weights the scan takes as *input* (Sec. 3.2: the
weights are "learned and normalized" upstream of the scan), and rounds to the
storage dtype.  Both the CPU oracle's tests and the GPU tests / benchmark take
their inputs from here, so the two sides always see identical values.

The paper evaluates on ImageNet classifiers and SDXL latents (Sec. 5.2-5.3);
neither the data nor the weights are available offline, so these tensors stand
in for them: same shapes (stage width 96 at 56x56, 1024-channel 128x128
latents, 512x512 / 256x1024 long scans, a 28x28 training stage), standard
normal features, softmax-normalised weights, uniform gates.

Draw order, per (batch b, weight group g) slice, generator
``numpy.random.default_rng([seed, b, g])``:
    x[cpg,H,W] ~ N(0,1);  then for d = 0..3:  logits[3,H,W] ~ N(0,1)*logit_scale,
    lam[cpg,H,W] ~ U(0,1), u[cpg,H,W] ~ U(0,1);  finally gy[cpg,H,W] ~ N(0,1).
Slices are independent, so any subset of (b, g) can be produced alone and is
identical to the same slice of the full tensors.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

DIR_TB, DIR_BT, DIR_LR, DIR_RL = 0, 1, 2, 3


@dataclass(frozen=True)
class ScanConfig:
    name: str
    B: int
    C: int
    H: int
    W: int
    G: int
    dtype: str = "f32"          # storage dtype: "f32", "bf16" or "f16"
    dir_mask: int = 15          # bit d set = direction d runs
    logit_scale: float = 1.0
    seed: int = 0

    @property
    def cpg(self) -> int:
        return self.C // self.G

    @property
    def n_dirs(self) -> int:
        return bin(self.dir_mask).count("1")

    @property
    def pixel_channels(self) -> int:
        return self.B * self.C * self.H * self.W

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype in ("bf16", "f16") else 4

    def fwd_algorithmic_bytes(self, save_h: bool = False) -> int:
        """Compulsory traffic of one forward call: every distinct input element
        read once, every output element written once."""
        D = self.n_dirs
        per_pc = 2 + 2 * D + (D if save_h else 0)          # x, y, lam_d, u_d (, h_d)
        w_elems = D * self.B * self.G * 3 * self.H * self.W
        return (per_pc * self.pixel_channels + w_elems) * self.elem_bytes

    def bwd_algorithmic_bytes(self) -> int:
        D = self.n_dirs
        per_pc = 3 + 5 * D                                  # gy, x, gx; lam,u,h in; glam,gu out
        w_elems = 2 * D * self.B * self.G * 3 * self.H * self.W
        return (per_pc * self.pixel_channels + w_elems) * self.elem_bytes


# The workloads named by the benchmark definition (one per line of its list).
CONFIGS = {
    "unit16":      ScanConfig("unit16", 1, 8, 16, 16, 1, "f32", 1, 1.0, 0),
    "cls56":       ScanConfig("cls56", 64, 96, 56, 56, 8, "bf16", 15, 1.0, 1),
    "diff128":     ScanConfig("diff128", 2, 1024, 128, 128, 16, "bf16", 15, 3.0, 2),
    "long512":     ScanConfig("long512", 1, 512, 512, 512, 16, "bf16", 15, 1.0, 3),
    "long256x1024": ScanConfig("long256x1024", 1, 512, 256, 1024, 16, "bf16", 15, 1.0, 3),
    "train28_gc":  ScanConfig("train28_gc", 32, 192, 28, 28, 192, "f32", 15, 1.0, 4),
    "train28_g4":  ScanConfig("train28_g4", 32, 192, 28, 28, 4, "f32", 15, 1.0, 4),
    # not in the benchmark definition: the classification, diffusion-latent and high-resolution shapes as training steps (forward with
    # h_save + backward)
    "train56":     ScanConfig("train56", 64, 96, 56, 56, 8, "bf16", 15, 1.0, 7),
    "train128":    ScanConfig("train128", 2, 1024, 128, 128, 16, "bf16", 15, 3.0, 5),
    "train512":    ScanConfig("train512", 1, 512, 512, 512, 16, "bf16", 15, 1.0, 6),
    # the 1024x1024 shapes of the paper's scaling study (Sec. 5.1: B = 16, C = 8) and of high-resolution generation
    # (App. B: 1152 channels); group counts are not stated there
    "scale1024":   ScanConfig("scale1024", 16, 8, 1024, 1024, 1, "f32", 15, 1.0, 9),
    "hires1024":   ScanConfig("hires1024", 1, 1152, 1024, 1024, 16, "bf16", 15, 1.0, 10),
    "hires2048":   ScanConfig("hires2048", 1, 64, 2048, 2048, 4, "bf16", 15, 1.0, 11),
    # the low-occupancy shape of the paper's throughput table (Table 1: 128x128, B = 1, C = 32; the group count is not
    # stated there): fewer planes than the chip has compute units, where GSPN-local's stretches are the work items
    "occ128":      ScanConfig("occ128", 1, 32, 128, 128, 4, "f32", 15, 1.0, 8),
    "occ128_train": ScanConfig("occ128_train", 1, 32, 128, 128, 4, "f32", 15, 1.0, 8),
}


def shrink(cfg: ScanConfig, **kw) -> ScanConfig:
    return replace(cfg, **kw)


# ------------------------------------------------------------------ dtypes
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """fp64/fp32 values -> storage array (float32, or uint16 bit patterns of bf16 / IEEE binary16)."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    if dtype == "f16":
        # from fp32, like the bf16 branch (the generators draw fp32 values)
        return np.ascontiguousarray(np.asarray(a, dtype=np.float32).astype(np.float16)).view(np.uint16)
    raise ValueError(dtype)


def storage_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact upcast of a storage array to float64."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    if dtype == "f16":
        return np.ascontiguousarray(a, dtype=np.uint16).view(np.float16).astype(np.float64)
    raise ValueError(dtype)


# ------------------------------------------------------------------ weights
def normalise_logits(logits: np.ndarray, d: int) -> np.ndarray:
    """[..., 3, H, W] raw logits -> weights that are row-stochastic over the
    neighbours that exist: plane k addresses offset k-1 on the orthogonal axis
    (columns for d = 0, 1; rows for d = 2, 3); a neighbour outside the image
    gets weight exactly 0 and the remaining ones are renormalised (softmax with
    the missing logits at -inf), computed in fp64."""
    z = np.array(logits, dtype=np.float64)
    if d in (DIR_TB, DIR_BT):
        z[..., 0, :, 0] = -np.inf
        z[..., 2, :, -1] = -np.inf
    else:
        z[..., 0, 0, :] = -np.inf
        z[..., 2, -1, :] = -np.inf
    z = z - z.max(axis=-3, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-3, keepdims=True)


# ------------------------------------------------------------------ slices
def make_slice(cfg: ScanConfig, b: int, g: int, with_gy: bool = True) -> dict:
    """Storage-dtype tensors of one (batch, weight-group) slice.

    returns dict:  x [cpg,H,W], w [4,3,H,W], lam [4,cpg,H,W], u [4,cpg,H,W],
    gy [cpg,H,W]; arrays are float32 (dtype f32) or uint16 bf16 bits (bf16).
    """
    rng = np.random.default_rng([cfg.seed, b, g])
    cpg, H, W = cfg.cpg, cfg.H, cfg.W
    x = rng.standard_normal((cpg, H, W), dtype=np.float32)
    w = np.empty((4, 3, H, W), dtype=np.float64)
    lam = np.empty((4, cpg, H, W), dtype=np.float32)
    u = np.empty((4, cpg, H, W), dtype=np.float32)
    for d in range(4):
        logits = rng.standard_normal((3, H, W), dtype=np.float32) * np.float32(cfg.logit_scale)
        w[d] = normalise_logits(logits, d)
        lam[d] = rng.random((cpg, H, W), dtype=np.float32)
        u[d] = rng.random((cpg, H, W), dtype=np.float32)
    out = {"x": to_storage(x, cfg.dtype), "w": to_storage(w, cfg.dtype),
           "lam": to_storage(lam, cfg.dtype), "u": to_storage(u, cfg.dtype)}
    if with_gy:
        out["gy"] = to_storage(rng.standard_normal((cpg, H, W), dtype=np.float32), cfg.dtype)
    return out


def make_inputs(cfg: ScanConfig, with_gy: bool = True) -> dict:
    """Full storage-dtype tensors: x [B,C,H,W], w [4,B,G,3,H,W],
    lam,u [4,B,C,H,W], gy [B,C,H,W]."""
    B, C, H, W, G, cpg = cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, cfg.cpg
    st = np.float32 if cfg.dtype == "f32" else np.uint16
    out = {"x": np.empty((B, C, H, W), st), "w": np.empty((4, B, G, 3, H, W), st),
           "lam": np.empty((4, B, C, H, W), st), "u": np.empty((4, B, C, H, W), st)}
    if with_gy:
        out["gy"] = np.empty((B, C, H, W), st)
    for b in range(B):
        for g in range(G):
            s = make_slice(cfg, b, g, with_gy)
            cs = slice(g * cpg, (g + 1) * cpg)
            out["x"][b, cs] = s["x"]
            out["w"][:, b, g] = s["w"]
            out["lam"][:, b, cs] = s["lam"]
            out["u"][:, b, cs] = s["u"]
            if with_gy:
                out["gy"][b, cs] = s["gy"]
    return out


def make_logits(cfg: ScanConfig) -> np.ndarray:
    """Raw weight logits [4, B, G, 3, H, W] ~ N(0, 1) * logit_scale in the storage dtype, for the calls that
    normalise inside (seeded by the config; nothing is masked: the taps that point outside a line are
    never read)."""
    rng = np.random.default_rng([cfg.seed, 977])
    z = rng.standard_normal((4, cfg.B, cfg.G, 3, cfg.H, cfg.W)) * cfg.logit_scale
    return to_storage(z, cfg.dtype)


def inputs_as_f64(inp: dict, dtype: str) -> dict:
    return {k: storage_to_f64(v, dtype) for k, v in inp.items()}
