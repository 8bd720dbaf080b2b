"""fp64 CPU oracle for the locally bi-directional selective scan.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing in the product package imports this
module, and this module imports nothing from the product package.

The arithmetic lives in ``lbscan_oracle.c`` (the scan) and ``conv1d_oracle.c``
(the block's pre-scan convolution), plain sequential C compiled with gcc; this
file only builds them and marshals numpy fp64 arrays through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "lbscan_oracle.c"), os.path.join(_HERE, "conv1d_oracle.c")]
_LIB = os.path.join(_HERE, "liblbscan_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)


class _Problem(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int), ("dim", ctypes.c_int), ("dstate", ctypes.c_int),
        ("seqlen", ctypes.c_int), ("window", ctypes.c_int),
        ("delta_softplus", ctypes.c_int),
        ("x", _dp), ("delta", _dp), ("A", _dp), ("Bm", _dp), ("Cm", _dp),
        ("Dskip", _dp), ("z", _dp), ("delta_bias", _dp),
    ]


def build(force: bool = False) -> str:
    """Compile the C oracle into a shared object next to its source."""
    stale = (not os.path.exists(_LIB)) or any(os.path.getmtime(_LIB) < os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
               "-ffp-contract=off", "-o", _LIB, *_SRCS, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.lbscan_ref_fwd.restype = ctypes.c_int
        lib.lbscan_ref_fwd.argtypes = [ctypes.POINTER(_Problem), _dp]
        lib.lbscan_ref_bidir_fwd.restype = ctypes.c_int
        lib.lbscan_ref_bidir_fwd.argtypes = [ctypes.POINTER(_Problem), ctypes.POINTER(_Problem), _dp]
        lib.lbscan_ref_bwd.restype = ctypes.c_int
        lib.lbscan_ref_bwd.argtypes = [ctypes.POINTER(_Problem)] + [_dp] * 9
        lib.lbscan_ref_fwd_state.restype = ctypes.c_int
        lib.lbscan_ref_fwd_state.argtypes = [ctypes.POINTER(_Problem), _dp, _dp, _dp]
        lib.lbscan_ref_bwd_state.restype = ctypes.c_int
        lib.lbscan_ref_bwd_state.argtypes = [ctypes.POINTER(_Problem)] + [_dp] * 12
        ci = ctypes.c_int
        lib.lbconv_ref_fwd.restype = ci
        lib.lbconv_ref_fwd.argtypes = [ci] * 6 + [_dp] * 4
        lib.lbconv_ref_bwd.restype = ci
        lib.lbconv_ref_bwd.argtypes = [ci] * 6 + [_dp] * 7
        lib.lbscan_ref_num_threads.restype = ctypes.c_int
        lib.lbscan_ref_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().lbscan_ref_num_threads())


def set_num_threads(n: int) -> None:
    _load().lbscan_ref_set_num_threads(int(n))


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_dp)


def _problem(x, delta, A, Bm, Cm, Dskip, z, delta_bias, window, delta_softplus):
    x, delta, A, Bm, Cm = (_f64(v) for v in (x, delta, A, Bm, Cm))
    Dskip, z, delta_bias = (_f64(v) for v in (Dskip, z, delta_bias))
    Bsz, D, L = x.shape
    N = A.shape[1]
    assert delta.shape == (Bsz, D, L) and A.shape == (D, N)
    assert Bm.shape == (Bsz, N, L) and Cm.shape == (Bsz, N, L)
    assert Dskip is None or Dskip.shape == (D,)
    assert delta_bias is None or delta_bias.shape == (D,)
    assert z is None or z.shape == (Bsz, D, L)
    keep = (x, delta, A, Bm, Cm, Dskip, z, delta_bias)
    p = _Problem(Bsz, D, N, L, int(window), int(bool(delta_softplus)),
                 _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm),
                 _ptr(Dskip), _ptr(z), _ptr(delta_bias))
    return p, keep


def fwd(x, delta, A, Bm, Cm, Dskip=None, z=None, delta_bias=None, *, window,
        delta_softplus=True, h0=None, return_state=False):
    """Locally bi-directional scan, forward.  Returns out (B,D,L) fp64, or
    (out, hT) with return_state.  h0 (B,D,N): forward state entering at step 0."""
    p, keep = _problem(x, delta, A, Bm, Cm, Dskip, z, delta_bias, window, delta_softplus)
    out = np.empty(keep[0].shape, dtype=np.float64)
    if h0 is None and not return_state:
        rc = _load().lbscan_ref_fwd(ctypes.byref(p), _ptr(out))
        if rc:
            raise RuntimeError(f"lbscan_ref_fwd failed: {rc}")
        return out
    Bsz, D, _ = keep[0].shape
    N = keep[2].shape[1]
    h0 = _f64(h0)
    assert h0 is None or h0.shape == (Bsz, D, N)
    hT = np.empty((Bsz, D, N), dtype=np.float64)
    rc = _load().lbscan_ref_fwd_state(ctypes.byref(p), _ptr(h0), _ptr(out), _ptr(hT))
    if rc:
        raise RuntimeError(f"lbscan_ref_fwd_state failed: {rc}")
    return (out, hT) if return_state else out


def bidir_fwd(set_f: dict, set_b: dict):
    """Global bi-directional scan (two full scans).  Each set is a dict with
    keys x, delta, A, Bm, Cm and optional Dskip, z, delta_bias, delta_softplus;
    the gate is taken from set_f."""
    def mk(s):
        return _problem(s["x"], s["delta"], s["A"], s["Bm"], s["Cm"], s.get("Dskip"),
                        s.get("z"), s.get("delta_bias"), 1, s.get("delta_softplus", True))
    pf, kf = mk(set_f)
    pb, kb = mk(set_b)
    out = np.empty(kf[0].shape, dtype=np.float64)
    rc = _load().lbscan_ref_bidir_fwd(ctypes.byref(pf), ctypes.byref(pb), _ptr(out))
    if rc:
        raise RuntimeError(f"lbscan_ref_bidir_fwd failed: {rc}")
    return out


def bwd(x, delta, A, Bm, Cm, Dskip=None, z=None, delta_bias=None, *, dout, window,
        delta_softplus=True, h0=None, dhT=None):
    """Gradients of fwd.  Returns a dict of fp64 arrays: dx, ddelta, dz (None
    without a gate), dBm, dCm, dA, dDskip, ddelta_bias; with h0 or dhT (the
    gradient arriving at the final state) also dh0."""
    p, keep = _problem(x, delta, A, Bm, Cm, Dskip, z, delta_bias, window, delta_softplus)
    xs = keep[0]
    Bsz, D, L = xs.shape
    N = keep[2].shape[1]
    dout = _f64(dout)
    assert dout.shape == xs.shape
    g = {
        "dx": np.empty_like(xs), "ddelta": np.empty_like(xs),
        "dz": np.empty_like(xs) if keep[6] is not None else None,
        "dBm": np.empty((Bsz, N, L)), "dCm": np.empty((Bsz, N, L)),
        "dA": np.empty((D, N)), "dDskip": np.empty((D,)), "ddelta_bias": np.empty((D,)),
    }
    if h0 is None and dhT is None:
        rc = _load().lbscan_ref_bwd(ctypes.byref(p), _ptr(dout), _ptr(g["dx"]), _ptr(g["ddelta"]),
                                    _ptr(g["dz"]), _ptr(g["dBm"]), _ptr(g["dCm"]), _ptr(g["dA"]),
                                    _ptr(g["dDskip"]), _ptr(g["ddelta_bias"]))
        if rc:
            raise RuntimeError(f"lbscan_ref_bwd failed: {rc}")
        return g
    h0, dhT = _f64(h0), _f64(dhT)
    assert h0 is None or h0.shape == (Bsz, D, N)
    assert dhT is None or dhT.shape == (Bsz, D, N)
    g["dh0"] = np.empty((Bsz, D, N))
    rc = _load().lbscan_ref_bwd_state(ctypes.byref(p), _ptr(h0), _ptr(dout), _ptr(dhT),
                                      _ptr(g["dx"]), _ptr(g["ddelta"]), _ptr(g["dz"]),
                                      _ptr(g["dBm"]), _ptr(g["dCm"]), _ptr(g["dA"]),
                                      _ptr(g["dDskip"]), _ptr(g["ddelta_bias"]), _ptr(g["dh0"]))
    if rc:
        raise RuntimeError(f"lbscan_ref_bwd_state failed: {rc}")
    return g


def conv1d_fwd(x, weight, bias=None, *, activation=True, reverse=False):
    """Depthwise causal convolution along the last axis, then SiLU (pre-scan step
    of the block).  x (B,D,L), weight (D,K), bias (D).  Returns y (B,D,L) fp64."""
    x, weight, bias = _f64(x), _f64(weight), _f64(bias)
    Bsz, D, L = x.shape
    K = weight.shape[1]
    assert weight.shape == (D, K) and (bias is None or bias.shape == (D,))
    y = np.empty_like(x)
    rc = _load().lbconv_ref_fwd(Bsz, D, L, K, int(bool(activation)), int(bool(reverse)),
                                _ptr(x), _ptr(weight), _ptr(bias), _ptr(y))
    if rc:
        raise RuntimeError(f"lbconv_ref_fwd failed: {rc}")
    return y


def conv1d_bwd(x, weight, bias=None, *, dy, activation=True, reverse=False):
    """Gradients of conv1d_fwd: dict with dx, dweight, dbias (None without bias)."""
    x, weight, bias, dy = _f64(x), _f64(weight), _f64(bias), _f64(dy)
    Bsz, D, L = x.shape
    K = weight.shape[1]
    assert dy.shape == x.shape
    g = {"dx": np.empty_like(x), "dweight": np.empty((D, K)),
         "dbias": np.empty((D,)) if bias is not None else None}
    rc = _load().lbconv_ref_bwd(Bsz, D, L, K, int(bool(activation)), int(bool(reverse)),
                                _ptr(x), _ptr(weight), _ptr(bias), _ptr(dy),
                                _ptr(g["dx"]), _ptr(g["dweight"]), _ptr(g["dbias"]))
    if rc:
        raise RuntimeError(f"lbconv_ref_bwd failed: {rc}")
    return g
