"""torch.autograd plumbing over the C ABI: the forward and backward entry points
wired into autograd.Function, so that the scan and the pre-scan convolution can sit
inside a PyTorch training step.  No arithmetic happens here: every value is
produced by the HIP kernels behind include/lbscan.h.
"""
from __future__ import annotations

import torch

from . import binding


class _LBScan(torch.autograd.Function):
    """out = lbscan_fwd(...); gradients from lbscan_bwd / lbscan_bwd_state.  The
    forward call leaves its state checkpoints in a saved_state buffer (when the
    library uses one for these shapes) and the backward call starts from them."""

    @staticmethod
    def forward(ctx, x, delta, A, Bm, Cm, Dskip, z, delta_bias, h0, window, delta_softplus, reverse,
                return_state):
        x, delta, Bm, Cm = (t.contiguous() for t in (x, delta, Bm, Cm))
        z = None if z is None else z.contiguous()
        saved = binding.lbscan_saved_state(x, A, window=window) if any(ctx.needs_input_grad) else None
        res = binding.lbscan_fwd(x, delta, A, Bm, Cm, Dskip, z, delta_bias, window=window,
                                 delta_softplus=delta_softplus, reverse=reverse, saved_state=saved,
                                 h0=h0, return_state=return_state)
        out, hT = res if return_state else (res, None)
        ctx.save_for_backward(x, delta, A, Bm, Cm, Dskip, z, delta_bias, h0, saved)
        ctx.cfg = (window, delta_softplus, reverse, return_state)
        if return_state:
            return out, hT
        return out

    @staticmethod
    def backward(ctx, dout, dhT=None):
        x, delta, A, Bm, Cm, Dskip, z, delta_bias, h0, saved = ctx.saved_tensors
        window, delta_softplus, reverse, return_state = ctx.cfg
        with_state = h0 is not None or (return_state and dhT is not None)
        g = binding.lbscan_bwd(x, delta, A, Bm, Cm, Dskip, z, delta_bias, dout=dout.contiguous(),
                               window=window, delta_softplus=delta_softplus, reverse=reverse,
                               saved_state=saved, h0=h0,
                               dhT=None if not with_state or dhT is None else dhT.contiguous())
        dh0 = g.get("dh0") if h0 is not None else None
        return (g["dx"], g["ddelta"], g["dA"], g["dBm"], g["dCm"], g["dDskip"], g["dz"],
                g["ddelta_bias"], dh0, None, None, None, None)


def lb_selective_scan(x, delta, A, Bm, Cm, Dskip=None, z=None, delta_bias=None, *, window,
                      delta_softplus=True, reverse=False, h0=None, return_state=False):
    """Differentiable locally bi-directional selective scan.  Shapes as in
    include/lbscan.h: x, delta, z (B,D,L); Bm, Cm (B,N,L); A (D,N), Dskip,
    delta_bias (D) and h0 (B,D,N) fp32.  Returns out, or (out, hT) with
    return_state."""
    return _LBScan.apply(x, delta, A, Bm, Cm, Dskip, z, delta_bias, h0, int(window),
                         bool(delta_softplus), bool(reverse), bool(return_state))


class _Conv1dSiLU(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, activation, reverse):
        x = x.contiguous()
        ctx.save_for_backward(x, weight, bias)
        ctx.cfg = (activation, reverse)
        return binding.lbscan_conv1d_fwd(x, weight, bias, activation=activation, reverse=reverse)

    @staticmethod
    def backward(ctx, dy):
        x, weight, bias = ctx.saved_tensors
        activation, reverse = ctx.cfg
        g = binding.lbscan_conv1d_bwd(x, weight, bias, dy=dy.contiguous(), activation=activation,
                                      reverse=reverse)
        return g["dx"], g["dweight"], g["dbias"], None, None


def causal_conv1d_silu(x, weight, bias=None, *, activation=True, reverse=False):
    """Differentiable pre-scan step: depthwise causal convolution along the last axis of
    x (B,D,L) with weight (D,K), K <= 4, bias (D), then SiLU."""
    return _Conv1dSiLU.apply(x, weight, bias, bool(activation), bool(reverse))
