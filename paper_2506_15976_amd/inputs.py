"""Seeded synthetic inputs for the locally bi-directional selective scan.

This module is shared by the GPU tests, the benchmark and the oracle tests.
It holds no arithmetic of the method itself: it only draws tensors with the
shapes and value distributions of the paper's workloads (Vim-tiny / Vim-small
token grids, a 1024x1024-image token grid, a MambaMIL whole-slide bag) and
rounds them to the storage type.  numpy only; it imports neither the HIP
binding nor the oracle.

Recipe (every workload): x, Bm, Cm, z, dout ~ N(0,1); raw delta = 0.5*N(0,1);
delta_bias[d] = log(expm1(dt_d)) with dt_d ~ U[1e-3, 0.1]; softplus on;
A[d,n] = -(n+1); Dskip = 1.  Draw order is fixed: x, delta, dt, Bm, Cm, z, dout.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20250615

# (batch, dim, dstate, seqlen, window, storage dtype, needs gradient)
WORKLOADS = {
    "tiny":       dict(batch=1,   dim=64,  dstate=16, seqlen=256,   window=4, dtype="fp32", grad=False, idx=0),
    "vim_tiny":   dict(batch=64,  dim=384, dstate=16, seqlen=197,   window=4, dtype="fp32", grad=False, idx=1),
    "vim_small":  dict(batch=128, dim=768, dstate=16, seqlen=197,   window=4, dtype="fp32", grad=True,  idx=2),
    "hires_4096": dict(batch=8,   dim=768, dstate=16, seqlen=4096,  window=8, dtype="bf16", grad=False, idx=3),
    "wsi_bag":    dict(batch=1,   dim=256, dstate=16, seqlen=65536, window=4, dtype="fp32", grad=True,  idx=4),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def fp32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) of values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_fp32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def make_inputs(batch, dim, dstate, seqlen, *, seed, dtype="fp32", with_z=True,
                with_dout=False, random_A=False):
    """Draw one input set.  Returns a dict of fp32 numpy arrays (values already
    rounded to bf16 when dtype == 'bf16'; A, Dskip, delta_bias always fp32)."""
    rng = np.random.default_rng(seed)
    B, D, N, L = batch, dim, dstate, seqlen
    x = rng.standard_normal((B, D, L), dtype=np.float32)
    delta = (0.5 * rng.standard_normal((B, D, L), dtype=np.float32)).astype(np.float32)
    dt = rng.uniform(1e-3, 0.1, size=(D,))
    Bm = rng.standard_normal((B, N, L), dtype=np.float32)
    Cm = rng.standard_normal((B, N, L), dtype=np.float32)
    z = rng.standard_normal((B, D, L), dtype=np.float32)
    dout = rng.standard_normal((B, D, L), dtype=np.float32) if with_dout else None
    if random_A:
        A = -rng.uniform(0.5, 16.0, size=(D, N)).astype(np.float32)
    else:
        A = -np.broadcast_to(np.arange(1, N + 1, dtype=np.float32), (D, N)).copy()
    s = dict(
        x=x, delta=delta, A=A, Bm=Bm, Cm=Cm,
        Dskip=np.ones((D,), dtype=np.float32),
        z=z if with_z else None,
        delta_bias=np.log(np.expm1(dt)).astype(np.float32),
        delta_softplus=True,
    )
    if dout is not None:
        s["dout"] = dout
    if dtype == "bf16":
        for k in ("x", "delta", "Bm", "Cm", "z", "dout"):
            if s.get(k) is not None:
                s[k] = round_to_bf16(s[k])
    elif dtype != "fp32":
        raise ValueError(f"unknown dtype {dtype!r}")
    return s


def make_workload(name: str, *, direction_b: bool = False):
    """Inputs of one named workload.  direction_b draws the independent second
    parameter set that the global bi-directional comparison scans backwards."""
    w = WORKLOADS[name]
    seed = BASE_SEED + w["idx"] + (1000 if direction_b else 0)
    s = make_inputs(w["batch"], w["dim"], w["dstate"], w["seqlen"], seed=seed,
                    dtype=w["dtype"], with_dout=w["grad"] and not direction_b)
    s["window"] = w["window"]
    return s


def column_order(seqlen: int, grid_h: int, grid_w: int, prefix: int = 0) -> np.ndarray:
    """Index array perm with scanned[j] = stored[perm[j]] for the column-by-column scan
    of a grid_h x grid_w token grid stored row by row at tokens [prefix, prefix + H W);
    tokens outside the grid keep their places.  (An index permutation only: the tests
    reorder inputs with it, run the oracle in plain sequence order and put the outputs
    back.)"""
    perm = np.arange(seqlen)
    hw = grid_h * grid_w
    assert prefix >= 0 and prefix + hw <= seqlen
    k = np.arange(hw)
    perm[prefix:prefix + hw] = prefix + (k % grid_h) * grid_w + k // grid_h
    return perm


def error_metric(got: np.ndarray, ref: np.ndarray, floor_frac: float = 0.1) -> float:
    """Scale-aware maximum relative error:
        max_i |got_i - ref_i| / max(|ref_i|, floor_frac * rms(ref)).
    A plain relative error is undefined where the reference crosses zero: each
    output is a sum of N+1 terms of size ~rms that may cancel, and fp32
    rounding of those terms leaves an absolute error of a few 1e-7 * rms on
    average and, in the tail over millions of outputs, up to ~1e-5 * rms (a
    sequential fp32 evaluation with correctly rounded exp shows the same).
    With the floor at 0.1 * rms a bound of 1e-4 therefore reads: relative
    error 1e-4 wherever the output is not a cancellation, absolute error
    1e-5 * rms where it is."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    floor = max(floor_frac * rms, 1e-300)
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def mean_error(got: np.ndarray, ref: np.ndarray) -> float:
    """Mean absolute error over rms(ref): catches a systematic loss of precision
    that the maximum, dominated by cancellations, would hide."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref))) or 1.0
    return float(np.mean(np.abs(got - ref)) / rms)
