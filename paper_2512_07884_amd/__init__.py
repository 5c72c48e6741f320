"""MI355X-native GSPN line-scan propagation (GSPN-2, Sec. 3.2 / 4): Python face of the C-ABI library.

The compute lives in ``libgspn.so`` (hand-written HIP for gfx950); this
package only marshals arguments.  Importing it is cheap; the shared library is
loaded on first use and a missing library raises (there is no CPU fallback).
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    if name in ("gspn_scan_fwd", "gspn_scan_bwd", "gspn_scan_fwd_local", "gspn_scan_bwd_local",
                "gspn_fwd_plan", "gspn_bwd_plan", "gspn_fwd_local_plan", "gspn_bwd_local_plan",
                "gspn_scan_fwd_logits", "gspn_scan_bwd_logits", "gspn_fwd_logits_plan", "gspn_bwd_logits_plan",
                "gspn_proxy_project", "gspn_proxy_project_bwd", "gspn_proxy_project_bwd_static", "gspn_proxy_plan", "gspn_scan_fwd_transposed", "gspn_fwd_transposed_plan",
                "gspn_scan_fwd_unfused", "gspn_unfused_workspace_bytes",
                "gspn_status_string", "gspn_version", "gspn_reload_env", "load_library", "lib_path", "GspnError"):
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
