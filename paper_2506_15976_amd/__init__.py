"""lbscan: locally bi-directional selective scan (LBMamba, arXiv 2506.15976) for MI355X.

The computation lives in hand-written HIP kernels behind a C ABI
(include/lbscan.h, paper_2506_15976_amd/csrc); this package is the thin Python
binding with the same entry-point names.
"""
from .binding import (  # noqa: F401
    LbscanArgs, LbscanConvArgs, LbscanError, lbscan_bidir_fwd, lbscan_bwd, lbscan_conv1d_bwd, lbscan_conv1d_fwd,
    lbscan_default_window, lbscan_fwd, lbscan_fwd_static, lbscan_saved_state, lbscan_set_option, lbscan_version,
    lbscan_workspace_bytes, load, make_args,
)
