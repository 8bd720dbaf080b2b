"""GPU parity of lbscan_bwd against the fp64 CPU oracle (itself pinned by finite
differences), every gradient, element by element, through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

GRADS = ("dx", "ddelta", "dz", "dBm", "dCm", "dA", "dDskip", "ddelta_bias")


@pytest.fixture(scope="module")
def lb():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2506_15976_amd as pkg
    pkg.load()
    return pkg


def _run_bwd(lb, oracle, s, *, window, dtype="fp32", reverse=False, softplus=True):
    import torch
    from gpu_util import assert_close, flip_time, fwd_inputs, to_device, to_numpy
    dev = to_device(s, dtype)
    got = lb.lbscan_bwd(**fwd_inputs(dev), dout=dev["dout"], window=window,
                        delta_softplus=softplus, reverse=reverse)
    torch.cuda.synchronize()
    src = flip_time(s) if reverse else s
    ref = oracle.bwd(**fwd_inputs(src), dout=src["dout"], window=window, delta_softplus=softplus)
    errs = {}
    for k in GRADS:
        r = ref[k]
        if r is None:
            assert got[k] is None
            continue
        if got[k] is None:
            # no gradient is produced for an optional input that was not given
            assert k in ("dDskip", "ddelta_bias") and s.get({"dDskip": "Dskip", "ddelta_bias": "delta_bias"}[k]) is None
            continue
        if reverse and r.ndim == 3:
            r = r[..., ::-1]
        errs[k] = assert_close(to_numpy(got[k]), r, dtype, k)
    return errs


@pytest.mark.parametrize("window", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("reverse", [False, True])
def test_tiny_workload_gradients(lb, oracle, window, reverse):
    from paper_2506_15976_amd.inputs import BASE_SEED, make_inputs
    s = make_inputs(1, 64, 16, 256, seed=BASE_SEED, with_dout=True)
    _run_bwd(lb, oracle, s, window=window, reverse=reverse)


@pytest.mark.parametrize("shape", [
    (2, 70, 16, 37), (1, 130, 16, 197), (3, 5, 16, 5), (2, 64, 16, 1), (2, 33, 16, 17),
    (1, 64, 8, 50), (2, 20, 3, 29), (1, 7, 1, 63),
])
@pytest.mark.parametrize("window", [1, 4, 8])
def test_ragged_shapes_gradients(lb, oracle, shape, window):
    from paper_2506_15976_amd.inputs import make_inputs
    B, D, N, L = shape
    s = make_inputs(B, D, N, L, seed=2234 + B * 7 + D + L, random_A=True, with_dout=True)
    _run_bwd(lb, oracle, s, window=window)
    _run_bwd(lb, oracle, s, window=window, reverse=True)


def test_gradients_without_optionals(lb, oracle):
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(2, 96, 16, 61, seed=177, with_z=False, with_dout=True)
    s["Dskip"] = None
    s["delta_bias"] = None
    _run_bwd(lb, oracle, s, window=4)
    s2 = make_inputs(2, 96, 16, 61, seed=178, with_dout=True)
    s2["delta"] = np.abs(s2["delta"]) * 0.2 + 0.01
    s2["delta_bias"] = None
    _run_bwd(lb, oracle, s2, window=4, softplus=False)


def test_gradients_bf16_storage(lb, oracle):
    from paper_2506_15976_amd.inputs import make_inputs
    for L in (64, 197, 33):
        s = make_inputs(2, 96, 16, L, seed=1300 + L, dtype="bf16", with_dout=True)
        _run_bwd(lb, oracle, s, window=8, dtype="bf16")


@pytest.mark.parametrize("L", [197, 193, 49])
def test_gradients_bf16_rows_of_odd_length(lb, oracle, L):
    """bf16 rows of odd length: the unaligned quad path of the tiles inside the rows,
    element accesses at the ragged tile and at the end of the last batch entry."""
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(3, 70, 16, L, seed=3400 + L, dtype="bf16", with_dout=True, random_A=True)
    for window in (4, 7):
        _run_bwd(lb, oracle, s, window=window, dtype="bf16")
        _run_bwd(lb, oracle, s, window=window, dtype="bf16", reverse=True)
    lb.lbscan_set_option("segments", 2)
    try:
        _run_bwd(lb, oracle, s, window=4, dtype="bf16")
    finally:
        lb.lbscan_set_option("segments", 0)


@pytest.mark.parametrize("segments", [2, 3, 5])
def test_gradients_with_rows_cut_into_segments(lb, oracle, segments):
    """Long rows are cut into segments in the backward pass too: forward carry
    chain for f, reverse chain for psi; force several cuts."""
    from paper_2506_15976_amd.inputs import make_inputs
    lb.lbscan_set_option("segments", segments)
    try:
        for (B, D, N, L, M) in [(1, 70, 16, 333, 4), (2, 64, 8, 160, 8), (1, 130, 16, 97, 16), (1, 64, 16, 700, 1)]:
            s = make_inputs(B, D, N, L, seed=7000 + D + L, random_A=True, with_dout=True)
            _run_bwd(lb, oracle, s, window=M)
            _run_bwd(lb, oracle, s, window=M, reverse=True)
        s = make_inputs(1, 96, 16, 256, seed=7100, dtype="bf16", with_dout=True)
        _run_bwd(lb, oracle, s, window=8, dtype="bf16")
        s = make_inputs(1, 64, 16, 300, seed=7200, with_z=False, with_dout=True)
        _run_bwd(lb, oracle, s, window=4)
    finally:
        lb.lbscan_set_option("segments", 0)


def test_long_rows_gradients_pick_segments_by_themselves(lb, oracle):
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(1, 64, 16, 5000, seed=7300, with_dout=True)
    _run_bwd(lb, oracle, s, window=4)
    _run_bwd(lb, oracle, s, window=16, reverse=True)


@pytest.mark.parametrize("name", ["vim_small", "wsi_bag"])
def test_full_size_gradients(lb, oracle, name):
    from paper_2506_15976_amd.inputs import WORKLOADS, make_workload
    w = WORKLOADS[name]
    s = make_workload(name)
    errs = _run_bwd(lb, oracle, s, window=w["window"], dtype=w["dtype"])
    print(name, {k: f"{v:.2e}" for k, v in errs.items()})


def test_saved_state_from_forward_gives_the_same_gradients(lb, oracle):
    """lbscan_fwd can leave checkpoints that lbscan_bwd starts from instead of
    recomputing them; both ways must agree with the oracle."""
    import torch
    from gpu_util import assert_close, flip_time, fwd_inputs, to_device, to_numpy
    from paper_2506_15976_amd.inputs import make_inputs
    lb.lbscan_set_option("segments", 1)      # small shapes would otherwise be cut into segments
    try:
        for (B, D, N, L, M, rev) in [(2, 130, 16, 197, 4, False), (3, 64, 16, 50, 8, True), (2, 70, 8, 33, 1, False)]:
            s = make_inputs(B, D, N, L, seed=8000 + L, random_A=True, with_dout=True)
            dev = to_device(s, "fp32")
            saved = lb.lbscan_saved_state(dev["x"], dev["A"], window=M)
            assert saved is not None
            saved.fill_(float("nan"))
            out = lb.lbscan_fwd(**fwd_inputs(dev), window=M, reverse=rev, saved_state=saved)
            got = lb.lbscan_bwd(**fwd_inputs(dev), dout=dev["dout"], window=M, reverse=rev, saved_state=saved)
            torch.cuda.synchronize()
            src = flip_time(s) if rev else s
            ref_out = oracle.fwd(**fwd_inputs(src), window=M)
            ref = oracle.bwd(**fwd_inputs(src), dout=src["dout"], window=M)
            assert_close(to_numpy(out), ref_out[..., ::-1] if rev else ref_out, "fp32", "out")
            for k in GRADS:
                r = ref[k][..., ::-1] if (rev and ref[k].ndim == 3) else ref[k]
                assert_close(to_numpy(got[k]), r, "fp32", k)
    finally:
        lb.lbscan_set_option("segments", 0)
    # long rows are cut into segments: no saved state for them
    big = to_device(make_inputs(1, 64, 16, 5000, seed=8100), "fp32")
    assert lb.lbscan_saved_state(big["x"], big["A"], window=4) is None


def test_missing_workspace_is_an_error(lb):
    import ctypes
    import torch
    from gpu_util import fwd_inputs, to_device
    from paper_2506_15976_amd.inputs import make_inputs
    dev = to_device(make_inputs(1, 64, 16, 64, seed=1, with_dout=True), "fp32")
    a = lb.make_args(**fwd_inputs(dev), window=4)
    o = {k: torch.empty_like(dev[v]) for k, v in (("dx", "x"), ("dd", "x"), ("dz", "x"), ("dB", "Bm"),
                                                  ("dC", "Cm"), ("dA", "A"), ("dD", "Dskip"), ("db", "delta_bias"))}
    rc = lb.load().lbscan_bwd(ctypes.byref(a), dev["dout"].data_ptr(), o["dx"].data_ptr(), o["dd"].data_ptr(),
                              o["dz"].data_ptr(), o["dB"].data_ptr(), o["dC"].data_ptr(), o["dA"].data_ptr(),
                              o["dD"].data_ptr(), o["db"].data_ptr(), None)
    assert rc == -3


def test_gradients_with_extreme_time_steps_and_decay_rates(lb, oracle):
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(2, 64, 16, 150, seed=9200, with_dout=True)
    r = np.random.default_rng(9201)
    s["delta"] = r.choice(np.array([-90.0, -12.0, -1.0, 0.5, 3.0, 25.0], dtype=np.float32),
                          size=s["delta"].shape).astype(np.float32)
    s["delta_bias"] = np.zeros_like(s["delta_bias"])
    s["A"] = -r.choice(np.array([1e-3, 0.5, 4.0, 40.0, 1e3], dtype=np.float32), size=s["A"].shape).astype(np.float32)
    for nseg in (0, 3):
        lb.lbscan_set_option("segments", nseg)
        try:
            _run_bwd(lb, oracle, s, window=4)
        finally:
            lb.lbscan_set_option("segments", 0)



@pytest.mark.parametrize("shape,window", [
    ((2, 70, 16, 37), 3), ((1, 130, 16, 197), 5), ((3, 5, 16, 50), 7), ((2, 64, 16, 64), 12),
    ((1, 64, 8, 100), 6), ((2, 20, 3, 29), 9), ((1, 7, 1, 63), 15), ((2, 64, 16, 10), 11),
    ((1, 66, 16, 131), 13), ((1, 64, 16, 48), 14),
])
@pytest.mark.parametrize("reverse", [False, True])
def test_gradients_any_window_up_to_a_tile(lb, oracle, shape, window, reverse):
    """Window lengths that 16 is not a multiple of: the backward kernel runs with
    run-time window masks and takes the adjoint of the local backward state that
    enters each 16-token tile from the summary pass."""
    from paper_2506_15976_amd.inputs import make_inputs
    B, D, N, L = shape
    s = make_inputs(B, D, N, L, seed=9400 + L + window, with_dout=True, random_A=True)
    _run_bwd(lb, oracle, s, window=window, reverse=reverse)


@pytest.mark.parametrize("nseg", [1, 3, 9])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_gradients_any_window_long_rows_in_segments(lb, oracle, nseg, dtype):
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(1, 70, 16, 601, seed=9420 + nseg, dtype=dtype, with_dout=True)
    lb.lbscan_set_option("segments", nseg)
    try:
        _run_bwd(lb, oracle, s, window=3, dtype=dtype)
        _run_bwd(lb, oracle, s, window=10, dtype=dtype, reverse=True)
    finally:
        lb.lbscan_set_option("segments", 0)


@pytest.mark.parametrize("shape,window", [
    ((2, 70, 16, 137), 17), ((1, 130, 16, 197), 24), ((1, 64, 16, 200), 32), ((2, 33, 8, 333), 100),
    ((1, 64, 16, 197), 196), ((1, 64, 16, 100), 99), ((1, 64, 16, 64), 48),
])
@pytest.mark.parametrize("reverse", [False, True])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_gradients_windows_longer_than_a_tile(lb, oracle, shape, window, reverse, dtype):
    """Sec. 3.2 leaves the window length free: windows longer than the 16-token tile
    (M < L), whose adjoint of the local backward state crosses tile boundaries."""
    from paper_2506_15976_amd.inputs import make_inputs
    B, D, N, L = shape
    s = make_inputs(B, D, N, L, seed=9500 + L + window, with_dout=True, random_A=True, dtype=dtype)
    _run_bwd(lb, oracle, s, window=window, reverse=reverse, dtype=dtype)


@pytest.mark.parametrize("nseg", [2, 5])
def test_gradients_long_windows_long_rows_in_segments(lb, oracle, nseg):
    """Segments are whole windows when windows straddle tile starts."""
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(1, 70, 16, 2000, seed=9520 + nseg, with_dout=True)
    lb.lbscan_set_option("segments", nseg)
    try:
        _run_bwd(lb, oracle, s, window=24)
        _run_bwd(lb, oracle, s, window=100, reverse=True)
        _run_bwd(lb, oracle, s, window=7)
    finally:
        lb.lbscan_set_option("segments", 0)
    _run_bwd(lb, oracle, s, window=40)          # default segmentation of a long row


def test_gradients_any_window_without_optionals_and_default_segments(lb, oracle):
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(1, 64, 16, 3000, seed=9430, with_dout=True, with_z=False)
    s["Dskip"] = None
    s["delta_bias"] = None
    _run_bwd(lb, oracle, s, window=6)


def test_full_size_gradients_bf16_4096_tokens(lb, oracle):
    """The 4096-token bf16 shape is a forward workload; its gradients are checked at
    full size too (M = 8 kernels, rows cut into segments, bf16 storage)."""
    from paper_2506_15976_amd.inputs import BASE_SEED, WORKLOADS, make_inputs
    w = WORKLOADS["hires_4096"]
    s = make_inputs(w["batch"], w["dim"], w["dstate"], w["seqlen"], seed=BASE_SEED + 53, dtype="bf16",
                    with_dout=True)
    errs = _run_bwd(lb, oracle, s, window=w["window"], dtype="bf16")
    print({k: f"{v:.2e}" for k, v in errs.items()})
