"""ctypes binding of liblbscan.so: argument marshalling only.

Every step of the computation runs in the HIP kernels behind the C ABI declared
in include/lbscan.h.  PyTorch is used for device memory and the current
stream, nothing else.  There is no CPU fallback: if the library has not been
built, loading fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblbscan.so")

LBSCAN_FP32, LBSCAN_BF16 = 0, 1
WS_FWD, WS_BWD, WS_BIDIR, WS_SAVED = 0, 1, 2, 3
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, -1, -2, -3, -4

EXPORTS = (
    "lbscan_fwd", "lbscan_bwd", "lbscan_bidir_fwd", "lbscan_workspace_bytes",
    "lbscan_default_window", "lbscan_strerror", "lbscan_last_error", "lbscan_version",
    "lbscan_set_option", "lbscan_bwd_state", "lbscan_conv1d_fwd", "lbscan_conv1d_bwd",
    "lbscan_fwd_static",
)


class LbscanArgs(ctypes.Structure):
    """Mirror of struct lbscan_args."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("dim", ctypes.c_int32), ("dstate", ctypes.c_int32),
        ("seqlen", ctypes.c_int32), ("window", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("delta_softplus", ctypes.c_int32), ("reverse", ctypes.c_int32),
        ("x", ctypes.c_void_p), ("delta", ctypes.c_void_p), ("Bm", ctypes.c_void_p),
        ("Cm", ctypes.c_void_p), ("z", ctypes.c_void_p), ("A", ctypes.c_void_p),
        ("Dskip", ctypes.c_void_p), ("delta_bias", ctypes.c_void_p), ("y", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("saved_state", ctypes.c_void_p), ("saved_state_bytes", ctypes.c_size_t),
        ("h0", ctypes.c_void_p), ("hT", ctypes.c_void_p),
        ("scan_order", ctypes.c_int32), ("grid_h", ctypes.c_int32), ("grid_w", ctypes.c_int32),
        ("grid_prefix", ctypes.c_int32),
    ]


class LbscanConvArgs(ctypes.Structure):
    """Mirror of struct lbscan_conv_args."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("dim", ctypes.c_int32), ("seqlen", ctypes.c_int32),
        ("width", ctypes.c_int32), ("dtype", ctypes.c_int32), ("activation", ctypes.c_int32),
        ("reverse", ctypes.c_int32),
        ("x", ctypes.c_void_p), ("weight", ctypes.c_void_p), ("bias", ctypes.c_void_p),
        ("y", ctypes.c_void_p),
    ]


class LbscanError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(what)


_lib = None


def load():
    """Load liblbscan.so (once).  torch is imported first so that the library
    binds to the HIP runtime already in the process."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2506_15976_amd.build` "
            "(there is no CPU fallback)")
    import torch  # noqa: F401  (loads libamdhip64 first)
    lib = ctypes.CDLL(LIB_PATH)
    ap = ctypes.POINTER(LbscanArgs)
    vp = ctypes.c_void_p
    lib.lbscan_fwd.restype = ctypes.c_int
    lib.lbscan_fwd.argtypes = [ap, vp]
    lib.lbscan_fwd_static.restype = ctypes.c_int
    lib.lbscan_fwd_static.argtypes = [ap, vp]
    lib.lbscan_bidir_fwd.restype = ctypes.c_int
    lib.lbscan_bidir_fwd.argtypes = [ap, ap, vp]
    lib.lbscan_bwd.restype = ctypes.c_int
    lib.lbscan_bwd.argtypes = [ap] + [vp] * 10
    lib.lbscan_bwd_state.restype = ctypes.c_int
    lib.lbscan_bwd_state.argtypes = [ap] + [vp] * 12
    cp = ctypes.POINTER(LbscanConvArgs)
    lib.lbscan_conv1d_fwd.restype = ctypes.c_int
    lib.lbscan_conv1d_fwd.argtypes = [cp, vp]
    lib.lbscan_conv1d_bwd.restype = ctypes.c_int
    lib.lbscan_conv1d_bwd.argtypes = [cp] + [vp] * 5
    lib.lbscan_workspace_bytes.restype = ctypes.c_size_t
    lib.lbscan_workspace_bytes.argtypes = [ap, ctypes.c_int]
    lib.lbscan_default_window.restype = ctypes.c_int
    lib.lbscan_default_window.argtypes = [ctypes.c_int32]
    lib.lbscan_set_option.restype = ctypes.c_int
    lib.lbscan_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int]
    lib.lbscan_strerror.restype = ctypes.c_char_p
    lib.lbscan_strerror.argtypes = [ctypes.c_int]
    lib.lbscan_last_error.restype = ctypes.c_char_p
    lib.lbscan_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(rc: int, name: str):
    if rc != OK:
        lib = load()
        msg = lib.lbscan_strerror(rc).decode()
        if rc == EHIP or (rc == EWORKSPACE and name.endswith("_static")):
            msg += ": " + lib.lbscan_last_error().decode()
        raise LbscanError(rc, f"{name} failed ({rc}): {msg}")


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return LBSCAN_FP32
    if t.dtype == torch.bfloat16:
        return LBSCAN_BF16
    raise LbscanError(EUNSUPPORTED, f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


ORDER_SEQUENCE, ORDER_COLUMNS = 0, 1


def make_args(x, delta, A, Bm, Cm, Dskip=None, z=None, delta_bias=None, *, window,
              delta_softplus=True, reverse=False, y=None, workspace=None, saved_state=None,
              h0=None, hT=None, grid=None):
    """Fill a struct lbscan_args from device tensors.  Shapes: x, delta, z, y
    (B,D,L); Bm, Cm (B,N,L); A (D,N) fp32; Dskip, delta_bias (D) fp32; h0, hT
    (B,D,N) fp32.  grid = (H, W) or (H, W, prefix): scan the H x W token grid that
    starts at token `prefix` column by column (see include/lbscan.h)."""
    import torch
    Bsz, D, L = x.shape
    N = A.shape[1]
    code = _dtype_code(x)
    for name, t, shape in (("delta", delta, (Bsz, D, L)), ("Bm", Bm, (Bsz, N, L)),
                           ("Cm", Cm, (Bsz, N, L)), ("z", z, (Bsz, D, L)), ("y", y, (Bsz, D, L))):
        if t is None:
            continue
        if tuple(t.shape) != shape or t.dtype != x.dtype:
            raise LbscanError(EINVAL, f"{name}: expected {shape} {x.dtype}, got {tuple(t.shape)} {t.dtype}")
    for name, t, shape in (("A", A, (D, N)), ("Dskip", Dskip, (D,)), ("delta_bias", delta_bias, (D,)),
                           ("h0", h0, (Bsz, D, N)), ("hT", hT, (Bsz, D, N))):
        if t is None:
            continue
        if tuple(t.shape) != shape or t.dtype != torch.float32:
            raise LbscanError(EINVAL, f"{name}: expected {shape} float32")
    for name, t in (("x", x), ("delta", delta), ("A", A), ("Bm", Bm), ("Cm", Cm), ("Dskip", Dskip),
                    ("z", z), ("delta_bias", delta_bias), ("y", y), ("workspace", workspace),
                    ("saved_state", saved_state), ("h0", h0), ("hT", hT)):
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise LbscanError(EINVAL, f"{name} must be a contiguous device tensor")
    a = LbscanArgs(Bsz, D, N, L, int(window), code, int(bool(delta_softplus)), int(bool(reverse)),
                   _ptr(x), _ptr(delta), _ptr(Bm), _ptr(Cm), _ptr(z), _ptr(A), _ptr(Dskip),
                   _ptr(delta_bias), _ptr(y), _ptr(workspace),
                   0 if workspace is None else workspace.numel() * workspace.element_size(),
                   _ptr(saved_state),
                   0 if saved_state is None else saved_state.numel() * saved_state.element_size(),
                   _ptr(h0), _ptr(hT))
    if grid is not None:
        a.scan_order = ORDER_COLUMNS
        a.grid_h, a.grid_w = int(grid[0]), int(grid[1])
        a.grid_prefix = int(grid[2]) if len(grid) > 2 else 0
    return a


def lbscan_workspace_bytes(args: LbscanArgs, which: int) -> int:
    return int(load().lbscan_workspace_bytes(ctypes.byref(args), which))


def lbscan_default_window(seqlen: int) -> int:
    return int(load().lbscan_default_window(seqlen))


def lbscan_set_option(name: str, value: int) -> None:
    _check(load().lbscan_set_option(name.encode(), int(value)), "lbscan_set_option")


def lbscan_version() -> str:
    return load().lbscan_version().decode()


def _workspace_for(args, which, like, stream=None):
    """Scratch for one call.  It is allocated from torch's caching allocator on the
    current stream; when the call runs on another stream the block is tied to that
    stream as well, so that it is not handed out again while the kernels use it."""
    import torch
    need = lbscan_workspace_bytes(args, which)
    if need == 0:
        return None
    ws = torch.empty((need + 3) // 4, dtype=torch.float32, device=like.device)
    _tie_to_stream(stream, ws)
    args.workspace = ws.data_ptr()
    args.workspace_bytes = ws.numel() * 4
    return ws


def _tie_to_stream(stream, *tensors):
    """Tensors this binding allocated (current stream) and hands to kernels that run
    on `stream`: record the use, so that the caching allocator waits for it."""
    if stream is None:
        return
    for t in tensors:
        if t is not None:
            t.record_stream(stream)


def _check_like(name, t, like):
    """Gradient / output tensors handed in by the caller: same shape, dtype, device
    kind and layout as the tensor they belong to."""
    if (tuple(t.shape) != tuple(like.shape) or t.dtype != like.dtype or not t.is_cuda
            or not t.is_contiguous()):
        raise LbscanError(EINVAL, f"{name} must be a contiguous device tensor of shape "
                                  f"{tuple(like.shape)} and dtype {like.dtype}")


def lbscan_saved_state(x, A, *, window):
    """Buffer for lbscan_fwd(saved_state=...) / lbscan_bwd(saved_state=...), or None
    when these shapes do not use one."""
    import torch
    a = LbscanArgs(x.shape[0], x.shape[1], A.shape[1], x.shape[2], int(window), _dtype_code(x))
    need = lbscan_workspace_bytes(a, WS_SAVED)
    return torch.empty((need + 3) // 4, dtype=torch.float32, device=x.device) if need else None


def lbscan_fwd(x, delta, A, Bm, Cm, Dskip=None, z=None, delta_bias=None, *, window,
               delta_softplus=True, reverse=False, out=None, stream=None, saved_state=None,
               h0=None, return_state=False, grid=None):
    """out = locally bi-directional scan of the inputs (see include/lbscan.h).
    h0 (B,D,N) fp32: forward state entering the call; with return_state the result
    is (out, hT), hT the state that leaves it."""
    import torch
    y = torch.empty_like(x) if out is None else out
    hT = None
    if return_state:
        hT = torch.empty((x.shape[0], x.shape[1], A.shape[1]), dtype=torch.float32, device=x.device)
    a = make_args(x, delta, A, Bm, Cm, Dskip, z, delta_bias, window=window,
                  delta_softplus=delta_softplus, reverse=reverse, y=y, saved_state=saved_state,
                  h0=h0, hT=hT, grid=grid)
    ws = _workspace_for(a, WS_FWD, x, stream)
    _tie_to_stream(stream, y if out is None else None, hT)
    _check(load().lbscan_fwd(ctypes.byref(a), _stream(stream)), "lbscan_fwd")
    del ws
    return (y, hT) if return_state else y


STATIC_SCRATCH_BYTES = 8 << 20


def lbscan_fwd_static(x, delta, A, Bm, Cm, Dskip=None, z=None, delta_bias=None, *, out, window,
                      delta_softplus=True, reverse=False, stream=None, h0=None, hT=None):
    """lbscan_fwd without any allocation: the caller passes every output (out, and hT
    if wanted); scratch is the library's fixed device array (see include/lbscan.h)."""
    a = make_args(x, delta, A, Bm, Cm, Dskip, z, delta_bias, window=window,
                  delta_softplus=delta_softplus, reverse=reverse, y=out, h0=h0, hT=hT)
    _check(load().lbscan_fwd_static(ctypes.byref(a), _stream(stream)), "lbscan_fwd_static")
    return out


def lbscan_bidir_fwd(set_f: dict, set_b: dict, *, out=None, stream=None):
    """Global bi-directional scan in two passes.  Each set is a dict with keys
    x, delta, A, Bm, Cm and optional Dskip, z, delta_bias, delta_softplus; the
    gate is set_f['z']."""
    import torch
    y = torch.empty_like(set_f["x"]) if out is None else out

    def mk(s, yy):
        return make_args(s["x"], s["delta"], s["A"], s["Bm"], s["Cm"], s.get("Dskip"), s.get("z"),
                         s.get("delta_bias"), window=1,
                         delta_softplus=s.get("delta_softplus", True), y=yy)
    af, ab = mk(set_f, y), mk(set_b, None)
    ws = _workspace_for(af, WS_BIDIR, y, stream)
    _tie_to_stream(stream, y if out is None else None)
    _check(load().lbscan_bidir_fwd(ctypes.byref(af), ctypes.byref(ab), _stream(stream)),
           "lbscan_bidir_fwd")
    del ws
    return y


def lbscan_bwd(x, delta, A, Bm, Cm, Dskip=None, z=None, delta_bias=None, *, dout, window,
               delta_softplus=True, reverse=False, stream=None, saved_state=None,
               h0=None, dhT=None, grid=None):
    """Gradients of lbscan_fwd.  Returns a dict: dx, ddelta, dz, dBm, dCm, dA,
    dDskip, ddelta_bias (None where the input is absent); with h0 or dhT (the
    gradient arriving at the state that left the forward call) also dh0, through
    lbscan_bwd_state."""
    import torch
    a = make_args(x, delta, A, Bm, Cm, Dskip, z, delta_bias, window=window,
                  delta_softplus=delta_softplus, reverse=reverse, saved_state=saved_state, h0=h0,
                  grid=grid)
    _check_like("dout", dout, x)
    g = dict(
        dx=torch.empty_like(x), ddelta=torch.empty_like(x),
        dz=torch.empty_like(x) if z is not None else None,
        dBm=torch.empty_like(Bm), dCm=torch.empty_like(Cm),
        dA=torch.empty_like(A),
        dDskip=torch.empty_like(Dskip) if Dskip is not None else None,
        ddelta_bias=torch.empty_like(delta_bias) if delta_bias is not None else None,
    )
    ws = _workspace_for(a, WS_BWD, x, stream)
    _tie_to_stream(stream, *g.values())
    if h0 is None and dhT is None:
        rc = load().lbscan_bwd(ctypes.byref(a), _ptr(dout), _ptr(g["dx"]), _ptr(g["ddelta"]),
                               _ptr(g["dz"]), _ptr(g["dBm"]), _ptr(g["dCm"]), _ptr(g["dA"]),
                               _ptr(g["dDskip"]), _ptr(g["ddelta_bias"]), _stream(stream))
        _check(rc, "lbscan_bwd")
    else:
        shape = (x.shape[0], x.shape[1], A.shape[1])
        if dhT is not None and (tuple(dhT.shape) != shape or dhT.dtype != torch.float32
                                or not dhT.is_cuda or not dhT.is_contiguous()):
            raise LbscanError(EINVAL, f"dhT must be a contiguous float32 device tensor of shape {shape}")
        g["dh0"] = torch.empty(shape, dtype=torch.float32, device=x.device)
        _tie_to_stream(stream, g["dh0"])
        rc = load().lbscan_bwd_state(ctypes.byref(a), _ptr(dout), _ptr(dhT), _ptr(g["dx"]),
                                     _ptr(g["ddelta"]), _ptr(g["dz"]), _ptr(g["dBm"]), _ptr(g["dCm"]),
                                     _ptr(g["dA"]), _ptr(g["dDskip"]), _ptr(g["ddelta_bias"]),
                                     _ptr(g["dh0"]), _stream(stream))
        _check(rc, "lbscan_bwd_state")
    del ws
    return g


def _conv_args(x, weight, bias, activation, reverse, y=None):
    import torch
    Bsz, D, L = x.shape
    K = weight.shape[1]
    if tuple(weight.shape) != (D, K) or weight.dtype != torch.float32:
        raise LbscanError(EINVAL, f"weight: expected ({D}, K) float32")
    if bias is not None and (tuple(bias.shape) != (D,) or bias.dtype != torch.float32):
        raise LbscanError(EINVAL, f"bias: expected ({D},) float32")
    for name, t in (("x", x), ("weight", weight), ("bias", bias), ("y", y)):
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise LbscanError(EINVAL, f"{name} must be a contiguous device tensor")
    return LbscanConvArgs(Bsz, D, L, K, _dtype_code(x), int(bool(activation)), int(bool(reverse)),
                          _ptr(x), _ptr(weight), _ptr(bias), _ptr(y))


def lbscan_conv1d_fwd(x, weight, bias=None, *, activation=True, reverse=False, out=None, stream=None):
    """y = SiLU(depthwise causal conv of x along the last axis) (see include/lbscan.h).
    x (B,D,L), weight (D,K) fp32 with K <= 4, bias (D) fp32."""
    import torch
    if out is not None:
        _check_like("out", out, x)
    y = torch.empty_like(x) if out is None else out
    _tie_to_stream(stream, y if out is None else None)
    a = _conv_args(x, weight, bias, activation, reverse, y)
    _check(load().lbscan_conv1d_fwd(ctypes.byref(a), _stream(stream)), "lbscan_conv1d_fwd")
    return y


def lbscan_conv1d_bwd(x, weight, bias=None, *, dy, activation=True, reverse=False, stream=None):
    """Gradients of lbscan_conv1d_fwd: dict with dx, dweight, dbias (None without bias)."""
    import torch
    _check_like("dy", dy, x)
    a = _conv_args(x, weight, bias, activation, reverse)
    g = dict(dx=torch.empty_like(x), dweight=torch.empty_like(weight),
             dbias=torch.empty_like(bias) if bias is not None else None)
    _tie_to_stream(stream, *g.values())
    rc = load().lbscan_conv1d_bwd(ctypes.byref(a), _ptr(dy), _ptr(g["dx"]), _ptr(g["dweight"]),
                                  _ptr(g["dbias"]), _stream(stream))
    _check(rc, "lbscan_conv1d_bwd")
    return g
