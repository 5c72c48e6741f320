"""The C-ABI library loads, exports what include/gspn.h declares, and rejects bad
arguments on the host (no kernel is launched by anything in this file)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2512_07884_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2512_07884_amd import build
        build.build(verbose=False)
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gspn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gspn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"gspn_scan_fwd", "gspn_scan_bwd", "gspn_status_string", "gspn_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    from paper_2512_07884_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_version_and_status_strings(lib):
    assert lib.gspn_version() >= 100
    seen = set()
    for s in range(0, 7):
        t = lib.gspn_status_string(s).decode()
        assert t and t != "unknown status"
        seen.add(t)
    assert len(seen) == 7
    assert lib.gspn_status_string(99).decode() == "unknown status"


def test_argument_errors_are_detected_before_any_launch(lib):
    p = ctypes.c_void_p(0x1000)          # aligned, never dereferenced: every call below fails validation
    bad = ctypes.c_void_p(0x1004)
    f = lambda *a, **k: lib.gspn_scan_fwd(*a)
    ok_dims = (1, 4, 8, 8, 2)
    assert lib.gspn_scan_fwd(None, p, p, p, p, None, *ok_dims, 15, 0, 0, None) == 1
    assert lib.gspn_scan_fwd(p, p, p, p, None, None, *ok_dims, 15, 0, 0, None) == 1
    assert lib.gspn_scan_fwd(p, p, p, p, p, None, 1, 4, 0, 8, 2, 15, 0, 0, None) == 2
    assert lib.gspn_scan_fwd(p, p, p, p, p, None, 1, 4, 8, 8, 3, 15, 0, 0, None) == 2      # C % G
    assert lib.gspn_scan_fwd(p, p, p, p, p, None, *ok_dims, 0, 0, 0, None) == 2
    assert lib.gspn_scan_fwd(p, p, p, p, p, None, *ok_dims, 16, 0, 0, None) == 2
    assert lib.gspn_scan_fwd(p, p, p, p, p, None, *ok_dims, 15, 3, 0, None) == 3          # dtype codes: 0 fp32, 1 bf16, 2 fp16
    assert lib.gspn_scan_fwd(p, p, p, p, p, None, *ok_dims, 15, -1, 0, None) == 3
    assert lib.gspn_scan_fwd(p, bad, p, p, p, None, *ok_dims, 15, 0, 0, None) == 4
    assert lib.gspn_scan_fwd(p, p, p, p, p, bad, *ok_dims, 15, 0, 0, None) == 4
    assert lib.gspn_scan_fwd(p, p, p, p, p, None, *ok_dims, 15, 0, 8, None) == 5           # unknown flag
    assert lib.gspn_scan_fwd(p, p, p, p, p, None, 1, 4, 8, 20000, 2, 15, 0, 0, None) == 5  # line too long
    assert lib.gspn_scan_bwd(p, p, p, p, p, None, p, p, p, p, *ok_dims, 15, 0, 0, None) == 1  # h_save required
    assert lib.gspn_scan_bwd(p, p, p, p, p, p, p, bad, p, p, *ok_dims, 15, 0, 0, None) == 4
    assert lib.gspn_scan_bwd(p, p, p, p, p, p, p, p, p, p, 1, 5, 8, 8, 2, 15, 0, 0, None) == 2
    # GSPN-local: the same checks, and a stretch of less than one line is a shape error
    assert lib.gspn_scan_fwd_local(p, p, p, p, p, None, *ok_dims, 0, 15, 0, 0, None) == 2
    assert lib.gspn_scan_fwd_local(p, p, p, p, p, None, *ok_dims, -3, 15, 0, 0, None) == 2
    assert lib.gspn_scan_fwd_local(None, p, p, p, p, None, *ok_dims, 4, 15, 0, 0, None) == 1
    assert lib.gspn_scan_fwd_local(p, p, p, p, p, bad, *ok_dims, 4, 15, 0, 0, None) == 4
    assert lib.gspn_scan_bwd_local(p, p, p, p, p, p, p, p, p, p, *ok_dims, 0, 15, 0, 0, None) == 2
    assert lib.gspn_scan_bwd_local(p, p, p, p, p, None, p, p, p, p, *ok_dims, 4, 15, 0, 0, None) == 1
    assert lib.gspn_scan_bwd_local(p, p, p, p, p, p, p, p, p, bad, *ok_dims, 4, 15, 0, 0, None) == 4


def test_logits_calls_check_their_arguments_and_dispatch_on_the_host(lib, monkeypatch):
    for v in ("GSPN_FORCE_GENERIC", "GSPN_FWD_NO_PLANE", "GSPN_BWD_NO_PLANE"):
        monkeypatch.delenv(v, raising=False)
    p = ctypes.c_void_p(0x1000)
    bad = ctypes.c_void_p(0x1008)
    dims = (1, 4, 8, 8, 2)
    big = 1 << 14
    assert lib.gspn_scan_fwd_logits(p, None, p, p, p, None, *dims, big, 15, 0, 0, None) == 1
    assert lib.gspn_scan_fwd_logits(p, p, p, p, p, None, *dims, 0, 15, 0, 0, None) == 2            # kchunk < 1
    assert lib.gspn_scan_fwd_logits(p, bad, p, p, p, None, *dims, big, 15, 0, 0, None) == 4
    assert lib.gspn_scan_fwd_logits(p, p, p, p, p, None, 1, 4, 8, 5000, 2, big, 15, 0, 0, None) == 5  # line too long here
    assert lib.gspn_scan_bwd_logits(p, p, p, p, p, None, p, p, p, p, *dims, big, 15, 0, 0, None) == 1
    assert lib.gspn_scan_bwd_logits(p, p, p, p, p, p, p, bad, p, p, *dims, big, 15, 0, 0, None) == 4
    assert lib.gspn_scan_bwd_logits(p, p, p, p, p, p, p, p, p, p, 1, 4, 5000, 8, 2, big, 15, 0, 0, None) == 5
    fwd = lambda *a: lib.gspn_fwd_logits_plan(*a).decode()
    bwd = lambda *a: lib.gspn_bwd_logits_plan(*a).decode()
    # dispatch as for the normalised weights (the training stage with per-channel weights is what the fusion is for)
    assert fwd(32, 192, 28, 28, 192, big, 15, 0, 0, 1) == "plane" and bwd(32, 192, 28, 28, 192, big, 15, 0, 0) == "plane"
    assert fwd(32, 192, 28, 28, 4, 7, 15, 0, 0, 1) == "plane" and bwd(32, 192, 28, 28, 4, 7, 15, 0, 0) == "plane"
    assert fwd(64, 96, 56, 56, 8, big, 15, 1, 0, 0) == "plane" and bwd(64, 96, 56, 56, 8, big, 15, 1, 0) == "twopass"
    assert fwd(2, 1024, 128, 128, 16, big, 15, 1, 0, 0) == "pair" and fwd(2, 1024, 128, 128, 16, big, 15, 0, 0, 0) == "tile" and fwd(1, 512, 512, 512, 16, big, 15, 1, 0, 0) == "stream"
    assert fwd(1, 2, 8, 5000, 1, big, 15, 0, 0, 0) == "invalid" and bwd(1, 2, 8, 8, 1, 0, 15, 0, 0) == "invalid"


def test_fp16_storage_dispatches_like_bf16_storage(lib, monkeypatch):
    for v in ("GSPN_FORCE_GENERIC", "GSPN_FWD_NO_PLANE", "GSPN_BWD_NO_PLANE", "GSPN_BWD_NO_TWOPASS", "GSPN_FWD_NO_PAIR", "GSPN_FWD_NO_CHUNK"):
        monkeypatch.delenv(v, raising=False)
    lib.gspn_reload_env()
    BF16, F16 = 1, 2
    for shape in ((2, 1024, 128, 128, 16), (1, 512, 512, 512, 16), (64, 96, 56, 56, 8), (32, 192, 28, 28, 4), (32, 192, 28, 28, 192),
                  (1, 8, 1024, 1024, 2), (1, 8, 33, 35, 2), (1, 3, 128, 128, 1), (2, 768, 7, 7, 8)):
        for has_h in (0, 1):
            assert lib.gspn_fwd_plan(*shape, 15, F16, 0, has_h) == lib.gspn_fwd_plan(*shape, 15, BF16, 0, has_h), shape
            assert lib.gspn_fwd_local_plan(*shape, 32, 15, F16, 0, has_h) == lib.gspn_fwd_local_plan(*shape, 32, 15, BF16, 0, has_h), shape
        assert lib.gspn_bwd_plan(*shape, 15, F16, 0) == lib.gspn_bwd_plan(*shape, 15, BF16, 0), shape
    assert lib.gspn_fwd_plan(2, 1024, 128, 128, 16, 15, F16, 0, 0).decode() == "pair"
    # the single-launch backward tile kernel exists in fp32 and bf16 storage: without the two passes fp16 goes generic
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    lib.gspn_reload_env()
    assert lib.gspn_bwd_plan(2, 8, 56, 56, 2, 15, BF16, 0).decode() == "tile" and lib.gspn_bwd_plan(2, 8, 56, 56, 2, 15, F16, 0).decode() == "generic"
    monkeypatch.delenv("GSPN_BWD_NO_TWOPASS")
    lib.gspn_reload_env()
    # the proxy projections run on the matrix cores in either 16-bit type
    assert lib.gspn_proxy_plan(2, 96, 8, 56, 56, F16).decode() == "mfma" and lib.gspn_proxy_plan(1, 12, 3, 5, 7, F16).decode() == "fma"
    assert lib.gspn_proxy_plan(1, 8, 4, 8, 8, 3).decode() == "invalid"


def test_plan_names(lib):
    assert lib.gspn_fwd_plan(1, 8, 16, 16, 1, 1, 0, 0, 0).decode() != "invalid"
    assert lib.gspn_fwd_plan(1, 8, 16, 16, 3, 1, 0, 0, 0).decode() == "invalid"
    assert lib.gspn_bwd_plan(32, 192, 28, 28, 4, 15, 0, 0).decode() != "invalid"


def test_kernel_family_chosen_for_local_scans(lib, monkeypatch):
    """GSPN-local dispatches like the global scan: every kernel family has its local instantiations."""
    for v in ("GSPN_FORCE_GENERIC", "GSPN_FWD_NO_PLANE", "GSPN_BWD_NO_PLANE", "GSPN_FWD_NO_CHUNK"):
        monkeypatch.delenv(v, raising=False)
    fwd = lambda *a: lib.gspn_fwd_local_plan(*a).decode()
    bwd = lambda *a: lib.gspn_bwd_local_plan(*a).decode()
    assert fwd(64, 96, 56, 56, 8, 14, 15, 1, 0, 0) == "plane" and bwd(32, 192, 28, 28, 4, 7, 15, 0, 0) == "plane"
    assert fwd(2, 1024, 128, 128, 16, 32, 15, 1, 0, 0) == "pair" and bwd(64, 96, 56, 56, 8, 14, 15, 1, 0) == "twopass"
    assert fwd(2, 1024, 128, 128, 16, 32, 15, 0, 0, 0) == "tile"
    assert fwd(1, 512, 512, 512, 16, 64, 15, 1, 0, 0) == "stream" and fwd(1, 2, 130, 67, 1, 9, 15, 0, 0, 0) == "generic"
    assert fwd(1, 8, 16, 16, 1, 0, 15, 0, 0, 0) == "invalid" and bwd(1, 8, 16, 16, 1, 0, 15, 0, 0) == "invalid"
    # few planes: the stretches are the work items (Sec. 4.1: the chunk index is part of the grid)
    assert fwd(1, 32, 128, 128, 4, 32, 15, 0, 0, 0) == "chunk" and fwd(1, 32, 128, 128, 4, 32, 15, 1, 0, 1) == "chunk"
    assert bwd(1, 32, 128, 128, 4, 32, 15, 0, 0) == "twopass"


def test_kernel_family_chosen_for_the_benchmark_shapes(lib, monkeypatch):
    """Host-side dispatch only: which kernel family each workload of the benchmark runs on."""
    for v in ("GSPN_FORCE_GENERIC", "GSPN_FWD_NO_PLANE", "GSPN_BWD_NO_PLANE", "GSPN_BWD_NO_TWOPASS", "GSPN_FWD_NO_PAIR"):
        monkeypatch.delenv(v, raising=False)
    fwd = lambda *a: lib.gspn_fwd_plan(*a).decode()
    bwd = lambda *a: lib.gspn_bwd_plan(*a).decode()
    assert fwd(1, 8, 16, 16, 1, 1, 0, 0, 0) == "plane"                       # unit16
    assert fwd(64, 96, 56, 56, 8, 15, 1, 0, 0) == "plane"                    # cls56
    assert fwd(2, 1024, 128, 128, 16, 15, 1, 0, 0) == "pair"                 # diff128
    assert fwd(1, 512, 512, 512, 16, 15, 1, 0, 0) == "stream"                # long512
    assert fwd(1, 512, 256, 1024, 16, 15, 1, 0, 0) == "stream"               # long256x1024
    assert fwd(16, 8, 1024, 1024, 1, 15, 0, 0, 0) == "stream"                # scale1024 (Sec. 5.1 scaling study)
    assert fwd(1, 1152, 1024, 1024, 16, 15, 1, 0, 0) == "stream"             # hires1024 (App. B)
    assert fwd(1, 64, 2048, 2048, 4, 15, 1, 0, 0) == "stream" and fwd(1, 8, 2048, 2048, 1, 15, 0, 0, 0) == "stream"
    assert bwd(16, 8, 1024, 1024, 1, 15, 0, 0) == "twopass" and bwd(1, 64, 2048, 2048, 4, 15, 1, 0) == "generic"
    for G in (192, 4):                                                        # train28_gc / train28_g4
        assert fwd(32, 192, 28, 28, G, 15, 0, 0, 1) == "plane"
        assert bwd(32, 192, 28, 28, G, 15, 0, 0) == "plane"
    assert bwd(64, 96, 56, 56, 8, 15, 1, 0) == "twopass" and bwd(64, 96, 56, 56, 8, 15, 0, 0) == "twopass"
    # the later stages of the paper's classifier (Sec. 5.2), forward with h_save and backward, both storage types
    for C, HW in ((192, 28), (384, 14), (768, 7)):
        for dt in (0, 1):
            assert fwd(64, C, HW, HW, 8, 15, dt, 0, 1) == "plane", (C, HW, dt)
            assert bwd(64, C, HW, HW, 8, 15, dt, 0) == ("twopass" if (HW, dt) == (28, 1) else "plane"), (C, HW, dt)   # (28x28 bf16: two passes measured faster)
    assert bwd(2, 1024, 128, 128, 16, 15, 1, 0) == "twopass"                 # beyond 64 lines: reverse sweep on the forward tile kernels + channel sum
    # training steps on the larger shapes: h_save on the stream kernel, two-pass backward (reverse sweep on the stream
    # kernel); small maps with one weight map per channel in bf16: two-pass with the reverse sweep on the plane kernel
    assert fwd(1, 512, 512, 512, 16, 15, 1, 0, 1) == "stream" and bwd(1, 512, 512, 512, 16, 15, 1, 0) == "twopass"
    assert bwd(64, 768, 7, 7, 768, 15, 1, 0) == "twopass" and bwd(64, 384, 14, 14, 384, 15, 1, 0) == "twopass"
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")                           # the kernels behind it stay reachable
    assert bwd(64, 96, 56, 56, 8, 15, 1, 0) == "tile" and bwd(2, 1024, 128, 128, 16, 15, 1, 0) == "generic"
    assert bwd(64, 192, 28, 28, 8, 15, 1, 0) == "plane"
    monkeypatch.delenv("GSPN_BWD_NO_TWOPASS")
    monkeypatch.setenv("GSPN_FORCE_GENERIC", "1")
    assert fwd(64, 96, 56, 56, 8, 15, 1, 0, 0) == "generic" and bwd(32, 192, 28, 28, 4, 15, 0, 0) == "generic"


def test_binding_refuses_cpu_tensors_and_missing_library(monkeypatch):
    import torch
    from paper_2512_07884_amd import binding
    x = torch.zeros(1, 2, 4, 4)
    with pytest.raises(ValueError):
        binding.gspn_scan_fwd(x, torch.zeros(4, 1, 1, 3, 4, 4), torch.zeros(4, 1, 2, 4, 4),
                              torch.zeros(4, 1, 2, 4, 4), torch.zeros(1, 2, 4, 4))
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "lib_path", lambda: "/nonexistent/libgspn.so")
    with pytest.raises(ImportError):
        binding.load_library()
