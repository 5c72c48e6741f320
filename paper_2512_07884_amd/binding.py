"""ctypes binding of libgspn.so: argument marshalling only.

Same entry-point names as include/gspn.h.  PyTorch tensors are used purely as
handles to device memory (``data_ptr()``) and for the current HIP stream; every
step of the scan runs in the library's kernels.  There is no CPU fallback: a
missing library raises, and so does any non-zero status from the library.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

GSPN_F32, GSPN_BF16, GSPN_F16 = 0, 1, 2
GSPN_FLAG_SHARED_PARAMS = 1
DIR_ALL = 15

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = ("gspn_scan_fwd", "gspn_scan_bwd", "gspn_scan_fwd_local", "gspn_scan_bwd_local",
           "gspn_scan_fwd_logits", "gspn_scan_bwd_logits",
           "gspn_fwd_plan", "gspn_bwd_plan", "gspn_fwd_local_plan", "gspn_bwd_local_plan",
           "gspn_fwd_logits_plan", "gspn_bwd_logits_plan", "gspn_proxy_project", "gspn_proxy_project_bwd", "gspn_proxy_project_bwd_static", "gspn_proxy_plan",
           "gspn_scan_fwd_transposed", "gspn_fwd_transposed_plan", "gspn_scan_fwd_unfused", "gspn_unfused_workspace_bytes",
           "gspn_status_string", "gspn_version", "gspn_reload_env")


class GspnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libgspn status {status}: {text}")
        self.status = status


def lib_path() -> str:
    """Path of the shared library; GSPN_LIBRARY overrides the in-tree build."""
    return os.environ.get("GSPN_LIBRARY") or os.path.join(_PKG, "libgspn.so")


def load_library() -> ctypes.CDLL:
    """Loads libgspn.so (built by ``python -m paper_2512_07884_amd.build``)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    # PyTorch ships its own HIP runtime; load it first so that libgspn binds to the
    # same runtime instance that owns the tensors and streams it will be handed.
    import torch  # noqa: F401
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2512_07884_amd.build` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(path)
    vp, ci, cu = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint
    lib.gspn_scan_fwd.argtypes = [vp] * 6 + [ci] * 5 + [cu, ci, cu, vp]
    lib.gspn_scan_fwd.restype = ci
    lib.gspn_scan_bwd.argtypes = [vp] * 10 + [ci] * 5 + [cu, ci, cu, vp]
    lib.gspn_scan_bwd.restype = ci
    lib.gspn_scan_fwd_local.argtypes = [vp] * 6 + [ci] * 6 + [cu, ci, cu, vp]
    lib.gspn_scan_fwd_local.restype = ci
    lib.gspn_scan_bwd_local.argtypes = [vp] * 10 + [ci] * 6 + [cu, ci, cu, vp]
    lib.gspn_scan_bwd_local.restype = ci
    lib.gspn_scan_fwd_logits.argtypes = [vp] * 6 + [ci] * 6 + [cu, ci, cu, vp]
    lib.gspn_scan_fwd_logits.restype = ci
    lib.gspn_scan_bwd_logits.argtypes = [vp] * 10 + [ci] * 6 + [cu, ci, cu, vp]
    lib.gspn_scan_bwd_logits.restype = ci
    lib.gspn_fwd_logits_plan.argtypes = [ci] * 6 + [cu, ci, cu, ci]
    lib.gspn_fwd_logits_plan.restype = ctypes.c_char_p
    lib.gspn_bwd_logits_plan.argtypes = [ci] * 6 + [cu, ci, cu]
    lib.gspn_bwd_logits_plan.restype = ctypes.c_char_p
    lib.gspn_scan_fwd_transposed.argtypes = [vp] * 6 + [ci] * 5 + [cu, ci, cu, vp]
    lib.gspn_scan_fwd_transposed.restype = ci
    lib.gspn_scan_fwd_unfused.argtypes = [vp] * 7 + [ctypes.c_ulonglong] + [ci] * 5 + [cu, ci, cu, vp]
    lib.gspn_scan_fwd_unfused.restype = ci
    lib.gspn_unfused_workspace_bytes.argtypes = [ci] * 4
    lib.gspn_unfused_workspace_bytes.restype = ctypes.c_ulonglong
    lib.gspn_fwd_transposed_plan.argtypes = [ci] * 5 + [cu, ci, cu]
    lib.gspn_fwd_transposed_plan.restype = ctypes.c_char_p
    lib.gspn_proxy_project.argtypes = [vp] * 3 + [ci] * 6 + [vp]
    lib.gspn_proxy_project.restype = ci
    lib.gspn_proxy_project_bwd.argtypes = [vp] * 6 + [ci] * 6 + [vp]
    lib.gspn_proxy_project_bwd.restype = ci
    lib.gspn_proxy_project_bwd_static.argtypes = [vp] * 5 + [ci] * 6 + [vp]
    lib.gspn_proxy_project_bwd_static.restype = ci
    lib.gspn_proxy_plan.argtypes = [ci] * 6
    lib.gspn_proxy_plan.restype = ctypes.c_char_p
    lib.gspn_fwd_local_plan.argtypes = [ci] * 6 + [cu, ci, cu, ci]
    lib.gspn_fwd_local_plan.restype = ctypes.c_char_p
    lib.gspn_bwd_local_plan.argtypes = [ci] * 6 + [cu, ci, cu]
    lib.gspn_bwd_local_plan.restype = ctypes.c_char_p
    lib.gspn_fwd_plan.argtypes = [ci] * 5 + [cu, ci, cu, ci]
    lib.gspn_fwd_plan.restype = ctypes.c_char_p
    lib.gspn_bwd_plan.argtypes = [ci] * 5 + [cu, ci, cu]
    lib.gspn_bwd_plan.restype = ctypes.c_char_p
    lib.gspn_status_string.argtypes = [ci]
    lib.gspn_status_string.restype = ctypes.c_char_p
    lib.gspn_version.argtypes = []
    lib.gspn_version.restype = ci
    lib.gspn_reload_env.argtypes = []
    lib.gspn_reload_env.restype = None
    _LIB = lib
    return lib


def gspn_status_string(status: int) -> str:
    return load_library().gspn_status_string(int(status)).decode()


def gspn_reload_env() -> None:
    """Makes the library read its GSPN_* environment variables again (it reads them once otherwise)."""
    load_library().gspn_reload_env()


def gspn_version() -> int:
    return int(load_library().gspn_version())


def gspn_fwd_plan(B, C, H, W, G, dir_mask=DIR_ALL, dtype=GSPN_F32, flags=0, has_h_save=False) -> str:
    return load_library().gspn_fwd_plan(B, C, H, W, G, dir_mask, dtype, flags, int(has_h_save)).decode()


def gspn_bwd_plan(B, C, H, W, G, dir_mask=DIR_ALL, dtype=GSPN_F32, flags=0) -> str:
    return load_library().gspn_bwd_plan(B, C, H, W, G, dir_mask, dtype, flags).decode()


def gspn_fwd_local_plan(B, C, H, W, G, kchunk, dir_mask=DIR_ALL, dtype=GSPN_F32, flags=0, has_h_save=False) -> str:
    return load_library().gspn_fwd_local_plan(B, C, H, W, G, kchunk, dir_mask, dtype, flags, int(has_h_save)).decode()


def gspn_bwd_local_plan(B, C, H, W, G, kchunk, dir_mask=DIR_ALL, dtype=GSPN_F32, flags=0) -> str:
    return load_library().gspn_bwd_local_plan(B, C, H, W, G, kchunk, dir_mask, dtype, flags).decode()


GLOBAL_SCAN = 1 << 14      # a kchunk no line reaches (GSPN_MAX_LINE): the global scan


def gspn_fwd_logits_plan(B, C, H, W, G, kchunk=GLOBAL_SCAN, dir_mask=DIR_ALL, dtype=GSPN_F32, flags=0, has_h_save=False) -> str:
    return load_library().gspn_fwd_logits_plan(B, C, H, W, G, kchunk, dir_mask, dtype, flags, int(has_h_save)).decode()


def gspn_bwd_logits_plan(B, C, H, W, G, kchunk=GLOBAL_SCAN, dir_mask=DIR_ALL, dtype=GSPN_F32, flags=0) -> str:
    return load_library().gspn_bwd_logits_plan(B, C, H, W, G, kchunk, dir_mask, dtype, flags).decode()


# ---------------------------------------------------------------- marshalling
def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return GSPN_F32
    if t.dtype == torch.bfloat16:
        return GSPN_BF16
    if t.dtype == torch.float16:
        return GSPN_F16
    raise TypeError(f"unsupported dtype {t.dtype}: float32, bfloat16 or float16")


def _ptr(t, name, shape, like):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name}: must be a device tensor")
    if t.device != like.device or t.dtype != like.dtype:
        raise ValueError(f"{name}: device/dtype differ from x")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)} != expected {tuple(shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status: int):
    if status != 0:
        raise GspnError(status, gspn_status_string(status))


def _fwd_args(x, w, lam, u, y, h_save, G, flags):
    B, C, H, W = x.shape
    if G is None:
        G = w.shape[2]
    slots = 1 if (flags & GSPN_FLAG_SHARED_PARAMS) else 4
    px = _ptr(x, "x", (B, C, H, W), x)
    pw = _ptr(w, "w", (slots, B, G, 3, H, W), x)
    pl = _ptr(lam, "lam", (slots, B, C, H, W), x)
    pu = _ptr(u, "u", (slots, B, C, H, W), x)
    py = _ptr(y, "y", (B, C, H, W), x)
    ph = _ptr(h_save, "h_save", (4, B, C, H, W), x)
    return [px, pw, pl, pu, py, ph], (B, C, H, W, G)


def gspn_scan_fwd(x, w, lam, u, y, h_save=None, *, G: Optional[int] = None, dir_mask: int = DIR_ALL,
                  flags: int = 0, stream=None) -> None:
    """y <- sum over directions of u_d * h_d (Eq. 1-2); optionally saves h_d.

    x [B,C,H,W]; w [4,B,G,3,H,W]; lam, u [4,B,C,H,W] ([1,...] with
    GSPN_FLAG_SHARED_PARAMS); y [B,C,H,W]; h_save [4,B,C,H,W] or None.
    All device tensors of one dtype (float32 / bfloat16 / float16), contiguous.
    """
    ptrs, dims = _fwd_args(x, w, lam, u, y, h_save, G, flags)
    _check(load_library().gspn_scan_fwd(*ptrs, *dims, dir_mask, _dtype_code(x), flags, _stream(stream)))


def gspn_scan_fwd_local(x, w, lam, u, y, h_save=None, *, kchunk: int, G: Optional[int] = None,
                        dir_mask: int = DIR_ALL, flags: int = 0, stream=None) -> None:
    """GSPN-local forward (Sec. 3.2): as gspn_scan_fwd, propagation confined to stretches of kchunk lines."""
    ptrs, dims = _fwd_args(x, w, lam, u, y, h_save, G, flags)
    _check(load_library().gspn_scan_fwd_local(*ptrs, *dims, int(kchunk), dir_mask, _dtype_code(x), flags,
                                              _stream(stream)))


def gspn_scan_fwd_logits(x, z, lam, u, y, h_save=None, *, kchunk: int = GLOBAL_SCAN, G: Optional[int] = None,
                         dir_mask: int = DIR_ALL, flags: int = 0, stream=None) -> None:
    """As gspn_scan_fwd with the weights given as raw logits z (softmax over the taps that exist, inside the call)."""
    ptrs, dims = _fwd_args(x, z, lam, u, y, h_save, G, flags)
    _check(load_library().gspn_scan_fwd_logits(*ptrs, *dims, int(kchunk), dir_mask, _dtype_code(x), flags,
                                               _stream(stream)))


def _bwd_args(gy, x, w, lam, u, h_save, gx, gw, glam, gu, G, flags):
    B, C, H, W = x.shape
    if G is None:
        G = w.shape[2]
    slots = 1 if (flags & GSPN_FLAG_SHARED_PARAMS) else 4
    args = [_ptr(gy, "gy", (B, C, H, W), x), _ptr(x, "x", (B, C, H, W), x),
            _ptr(w, "w", (slots, B, G, 3, H, W), x), _ptr(lam, "lam", (slots, B, C, H, W), x),
            _ptr(u, "u", (slots, B, C, H, W), x), _ptr(h_save, "h_save", (4, B, C, H, W), x),
            _ptr(gx, "gx", (B, C, H, W), x), _ptr(gw, "gw", (4, B, G, 3, H, W), x),
            _ptr(glam, "glam", (4, B, C, H, W), x), _ptr(gu, "gu", (4, B, C, H, W), x)]
    return args, (B, C, H, W, G)


def gspn_scan_bwd(gy, x, w, lam, u, h_save, gx, gw, glam, gu, *, G: Optional[int] = None,
                  dir_mask: int = DIR_ALL, flags: int = 0, stream=None) -> None:
    """Gradients of the forward scan (see include/gspn.h); outputs overwritten."""
    args, dims = _bwd_args(gy, x, w, lam, u, h_save, gx, gw, glam, gu, G, flags)
    _check(load_library().gspn_scan_bwd(*args, *dims, dir_mask, _dtype_code(x), flags, _stream(stream)))


def gspn_scan_bwd_local(gy, x, w, lam, u, h_save, gx, gw, glam, gu, *, kchunk: int, G: Optional[int] = None,
                        dir_mask: int = DIR_ALL, flags: int = 0, stream=None) -> None:
    """Gradients of the GSPN-local forward scan with the same kchunk; outputs overwritten."""
    args, dims = _bwd_args(gy, x, w, lam, u, h_save, gx, gw, glam, gu, G, flags)
    _check(load_library().gspn_scan_bwd_local(*args, *dims, int(kchunk), dir_mask, _dtype_code(x), flags,
                                              _stream(stream)))



def gspn_scan_bwd_logits(gy, x, z, lam, u, h_save, gx, gz, glam, gu, *, kchunk: int = GLOBAL_SCAN,
                         G: Optional[int] = None, dir_mask: int = DIR_ALL, flags: int = 0, stream=None) -> None:
    """Gradients of gspn_scan_fwd_logits; gz (shape of z) is the gradient w.r.t. the logits; outputs overwritten."""
    args, dims = _bwd_args(gy, x, z, lam, u, h_save, gx, gz, glam, gu, G, flags)
    _check(load_library().gspn_scan_bwd_logits(*args, *dims, int(kchunk), dir_mask, _dtype_code(x), flags,
                                               _stream(stream)))


def gspn_proxy_plan(B, K, M, H, W, dtype=GSPN_BF16) -> str:
    return load_library().gspn_proxy_plan(B, K, M, H, W, dtype).decode()


def gspn_proxy_project(inp, P, out, *, stream=None) -> None:
    """out[b, m] = sum_k P[m, k] * inp[b, k] per pixel (compressive proxy projection, Sec. 4.2).
    inp [B,K,H,W]; P [M,K]; out [B,M,H,W]; device tensors of one dtype, contiguous."""
    B, K, H, W = inp.shape
    M = P.shape[0]
    args = [_ptr(inp, "inp", (B, K, H, W), inp), _ptr(P, "P", (M, K), inp), _ptr(out, "out", (B, M, H, W), inp)]
    _check(load_library().gspn_proxy_project(*args, B, K, M, H, W, _dtype_code(inp), _stream(stream)))


def gspn_proxy_project_bwd(gout, inp, P, gin, gP, partial, *, stream=None) -> None:
    """Gradients of gspn_proxy_project: gin[b, k] = sum_m P[m, k] * gout[b, m] per pixel (storage dtype, or None) and
    gP[m, k] = sum over images and pixels of gout[b, m] * inp[b, k] (float32 [M,K], or None); partial: float32 [B,M,K]
    workspace, required with gP.  gout [B,M,H,W]; inp [B,K,H,W]; P [M,K]; device tensors, contiguous."""
    import torch
    B, K, H, W = inp.shape
    M = P.shape[0]
    args = [_ptr(gout, "gout", (B, M, H, W), inp), _ptr(inp, "inp", (B, K, H, W), inp), _ptr(P, "P", (M, K), inp),
            _ptr(gin, "gin", (B, K, H, W), inp)]
    for t, name, shape in ((gP, "gP", (M, K)), (partial, "partial", (B, M, K))):
        if t is None:
            args.append(None)
            continue
        if not t.is_cuda or t.device != inp.device or t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError(f"{name}: must be a contiguous float32 device tensor of shape {shape}")
        args.append(ctypes.c_void_p(t.data_ptr()))
    _check(load_library().gspn_proxy_project_bwd(*args, B, K, M, H, W, _dtype_code(inp), _stream(stream)))


def gspn_proxy_project_bwd_static(gout, inp, P, gin, gP, *, stream=None) -> None:
    """gspn_proxy_project_bwd without the workspace argument: the per-image sums go to a static device array of the
    library's (B*M*K <= 2**20 floats, else GspnError); the call allocates nothing.  Calls that overlap on one GPU race."""
    import torch
    B, K, H, W = inp.shape
    M = P.shape[0]
    args = [_ptr(gout, "gout", (B, M, H, W), inp), _ptr(inp, "inp", (B, K, H, W), inp), _ptr(P, "P", (M, K), inp),
            _ptr(gin, "gin", (B, K, H, W), inp)]
    if gP is None:
        args.append(None)
    else:
        if not gP.is_cuda or gP.device != inp.device or gP.dtype != torch.float32 or tuple(gP.shape) != (M, K) or not gP.is_contiguous():
            raise ValueError(f"gP: must be a contiguous float32 device tensor of shape {(M, K)}")
        args.append(ctypes.c_void_p(gP.data_ptr()))
    _check(load_library().gspn_proxy_project_bwd_static(*args, B, K, M, H, W, _dtype_code(inp), _stream(stream)))


def gspn_fwd_transposed_plan(B, C, H, W, G, dir_mask=DIR_ALL, dtype=GSPN_F32, flags=0) -> str:
    return load_library().gspn_fwd_transposed_plan(B, C, H, W, G, dir_mask, dtype, flags).decode()


def gspn_scan_fwd_transposed(x, xt, w, lam, u, y, *, G: Optional[int] = None, dir_mask: int = DIR_ALL, flags: int = 0,
                             stream=None) -> None:
    """Forward scan with the horizontal directions stored transposed: xt [B,C,W,H]; slots 2 and 3 of w, lam, u hold
    [B,G,3,W,H] / [B,C,W,H] in the same memory footprint as the untransposed slots (pass tensors of the usual shapes
    whose slots 2, 3 were filled through a transposed view).  y [B,C,H,W]."""
    B, C, H, W = x.shape
    if G is None:
        G = w.shape[2]
    slots = 1 if (flags & GSPN_FLAG_SHARED_PARAMS) else 4
    args = [_ptr(x, "x", (B, C, H, W), x), _ptr(xt, "xt", (B, C, W, H), x), _ptr(w, "w", (slots, B, G, 3, H, W), x),
            _ptr(lam, "lam", (slots, B, C, H, W), x), _ptr(u, "u", (slots, B, C, H, W), x), _ptr(y, "y", (B, C, H, W), x)]
    _check(load_library().gspn_scan_fwd_transposed(*args, B, C, H, W, G, dir_mask, _dtype_code(x), flags, _stream(stream)))


def gspn_unfused_workspace_bytes(B: int, C: int, H: int, W: int) -> int:
    return int(load_library().gspn_unfused_workspace_bytes(B, C, H, W))


def gspn_scan_fwd_unfused(x, w, lam, u, y, h_save, workspace, *, G: Optional[int] = None, dir_mask: int = DIR_ALL,
                          flags: int = 0, stream=None) -> None:
    """The comparator of the fused kernels: one launch per line and direction, the state handed on through global
    memory (`workspace`: a device tensor of at least gspn_unfused_workspace_bytes(B, C, H, W) bytes).  Never dispatched
    to by the other calls."""
    ptrs, (B, C, H, W, G) = _fwd_args(x, w, lam, u, y, h_save, G, flags)
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().gspn_scan_fwd_unfused(*ptrs, workspace.data_ptr(), nbytes, B, C, H, W, G, dir_mask,
                                                _dtype_code(x), flags, _stream(stream)))
