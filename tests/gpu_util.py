"""Helpers shared by the GPU parity tests: host<->device marshalling and the error norm."""
import numpy as np

from paper_2512_07884_amd import workloads as WL

# max|gpu - oracle| / max|oracle| per tensor.  fp16 storage: the bf16 bound scaled by the ratio of the two formats'
# rounding units (2^-11 against 2^-8 relative spacing): every rounding the kernels make is to storage, at the same points
TOL = {"f32": 1e-5, "bf16": 1e-2, "f16": 1.25e-3}
TORCH_16 = {"bf16": "bfloat16", "f16": "float16"}


def to_device(arr: np.ndarray, dtype: str):
    import torch
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.uint16).view(np.int16)).cuda().view(getattr(torch, TORCH_16[dtype]))


def to_host_f64(t) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def empty_like_dev(shape, dtype: str, fill=None):
    import torch
    td = torch.float32 if dtype == "f32" else getattr(torch, TORCH_16[dtype])
    t = torch.empty(shape, dtype=td, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def rel_inf_err(a: np.ndarray, ref: np.ndarray) -> float:
    scale = np.max(np.abs(ref))
    if scale == 0:
        return float(np.max(np.abs(a)))
    return float(np.max(np.abs(a - ref)) / scale)


def run_fwd_gpu(inp: dict, cfg, dir_mask=None, save_h=False, flags=0, poison=True):
    """inp: storage arrays from workloads.make_inputs (possibly with a 1-slot
    direction axis when flags has SHARED_PARAMS).  Returns y (and h) as float64."""
    import torch
    import paper_2512_07884_amd as G
    mask = cfg.dir_mask if dir_mask is None else dir_mask
    dev = {k: to_device(v, cfg.dtype) for k, v in inp.items() if k in ("x", "w", "lam", "u")}
    B, C, H, W = inp["x"].shape
    y = empty_like_dev((B, C, H, W), cfg.dtype, float("nan") if poison else None)
    hs = empty_like_dev((4, B, C, H, W), cfg.dtype, float("nan") if poison else None) if save_h else None
    G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, G=cfg.G, dir_mask=mask, flags=flags)
    torch.cuda.synchronize()
    return (to_host_f64(y), to_host_f64(hs) if save_h else None, dev, y, hs)
