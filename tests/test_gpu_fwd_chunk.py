"""GPU parity of the chunk-per-lane forward kernel (one wave per row, 16 tokens per
lane, prefix scan over the lanes) against the fp64 CPU oracle.  The kernel is picked
by the library for long rows that are many; here it is forced on small shapes too."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lb():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2506_15976_amd as pkg
    pkg.load()
    return pkg


@pytest.fixture()
def chunk_mapping(lb):
    lb.lbscan_set_option("mapping", 2)
    yield
    lb.lbscan_set_option("mapping", 0)


def _run_fwd(lb, oracle, s, *, window, dtype="fp32", softplus=True, reverse=False):
    import torch
    from gpu_util import assert_close, flip_time, fwd_inputs, to_device, to_numpy
    dev = to_device(s, dtype)
    got = lb.lbscan_fwd(**fwd_inputs(dev), window=window, delta_softplus=softplus, reverse=reverse)
    torch.cuda.synchronize()
    src = flip_time(s) if reverse else s
    ref = oracle.fwd(**fwd_inputs(src), window=window, delta_softplus=softplus)
    if reverse:
        ref = ref[..., ::-1]
    return assert_close(to_numpy(got), ref, dtype)


@pytest.mark.parametrize("window", [1, 2, 4, 8, 16])
def test_every_compiled_window(lb, oracle, chunk_mapping, window):
    from paper_2506_15976_amd.inputs import make_inputs
    # less than a chunk; a chunk and a ragged second one; rows that do not fill a block
    for (B, D, N, L) in [(2, 5, 16, 37), (1, 13, 16, 1500), (2, 8, 16, 1024)]:
        s = make_inputs(B, D, N, L, seed=7100 + D + L, random_A=True)
        _run_fwd(lb, oracle, s, window=window)
        _run_fwd(lb, oracle, s, window=window, reverse=True)


@pytest.mark.parametrize("shape", [
    (1, 9, 16, 2049), (2, 3, 8, 1023), (1, 17, 3, 1025), (1, 1, 1, 3100), (3, 8, 16, 1), (1, 20, 16, 4096),
])
def test_ragged_shapes_and_small_state_sizes(lb, oracle, chunk_mapping, shape):
    from paper_2506_15976_amd.inputs import make_inputs
    B, D, N, L = shape
    s = make_inputs(B, D, N, L, seed=7200 + D + L, random_A=True)
    _run_fwd(lb, oracle, s, window=4)
    _run_fwd(lb, oracle, s, window=8, reverse=True)
    s["delta"] = np.abs(s["delta"]) * 0.1          # used as the time step itself
    s["delta_bias"] = np.abs(s["delta_bias"]) * 0.1
    _run_fwd(lb, oracle, s, window=16, softplus=False)


def test_bf16_storage(lb, oracle, chunk_mapping):
    from paper_2506_15976_amd.inputs import make_inputs
    for (B, D, L, M) in [(2, 12, 1500, 8), (1, 8, 64, 4), (1, 9, 2050, 16)]:
        s = make_inputs(B, D, 16, L, seed=7300 + L, dtype="bf16")
        _run_fwd(lb, oracle, s, window=M, dtype="bf16")
        _run_fwd(lb, oracle, s, window=M, dtype="bf16", reverse=True)


def test_bf16_rows_of_odd_length_fall_back(lb, oracle, chunk_mapping):
    """Rows that start at odd bf16 elements allow no quad accesses: the row-per-lane
    kernels take the call, with the same result."""
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(1, 9, 16, 1501, seed=7310, dtype="bf16")
    _run_fwd(lb, oracle, s, window=4, dtype="bf16")


def test_optional_arguments_absent(lb, oracle, chunk_mapping):
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(1, 10, 16, 1300, seed=7400, random_A=True)
    for drop in (("z",), ("Dskip",), ("delta_bias",), ("z", "Dskip", "delta_bias")):
        t = dict(s)
        for k in drop:
            t[k] = None
        _run_fwd(lb, oracle, t, window=4)


def test_entering_and_leaving_states(lb, oracle, chunk_mapping):
    import torch
    from gpu_util import assert_close, fwd_inputs, to_device, to_numpy
    from paper_2506_15976_amd.inputs import make_inputs
    for (B, D, N, L) in [(2, 11, 16, 2300), (1, 8, 5, 100)]:
        s = make_inputs(B, D, N, L, seed=7500 + L, random_A=True)
        dev = to_device(s, "fp32")
        h0 = np.random.default_rng(7501).standard_normal((B, D, N)).astype(np.float32)
        out, hT = lb.lbscan_fwd(**fwd_inputs(dev), window=8, h0=torch.from_numpy(h0).cuda(), return_state=True)
        torch.cuda.synchronize()
        ref, ref_hT = oracle.fwd(**fwd_inputs(s), window=8, h0=h0, return_state=True)
        assert_close(to_numpy(out), ref, "fp32", "out")
        assert_close(to_numpy(hT), ref_hT, "fp32", "hT")
        # the reversed sequence: the state enters at the last stored token
        from gpu_util import flip_time
        out, hT = lb.lbscan_fwd(**fwd_inputs(dev), window=8, h0=torch.from_numpy(h0).cuda(), return_state=True,
                                reverse=True)
        torch.cuda.synchronize()
        ref, ref_hT = oracle.fwd(**fwd_inputs(flip_time(s)), window=8, h0=h0, return_state=True)
        assert_close(to_numpy(out), ref[..., ::-1], "fp32", "out, reversed")
        assert_close(to_numpy(hT), ref_hT, "fp32", "hT, reversed")


def test_extreme_time_steps_and_decay_rates(lb, oracle, chunk_mapping):
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(2, 16, 16, 1300, seed=7600)
    r = np.random.default_rng(7601)
    s["delta"] = r.choice(np.array([-90.0, -12.0, -1.0, 0.5, 3.0, 25.0], dtype=np.float32),
                          size=s["delta"].shape).astype(np.float32)
    s["delta_bias"] = np.zeros_like(s["delta_bias"])
    s["A"] = -r.choice(np.array([1e-3, 0.5, 4.0, 40.0, 1e3], dtype=np.float32), size=s["A"].shape).astype(np.float32)
    _run_fwd(lb, oracle, s, window=4)
    _run_fwd(lb, oracle, s, window=16)


def test_two_pass_comparison_and_any_window_through_this_kernel(lb, oracle, chunk_mapping):
    """The global bi-directional comparison (window-1 scan left to right into fp32, then
    right to left on top of it) and the first pass of the any-window path take the same
    kernel when it applies."""
    import torch
    from gpu_util import assert_close, fwd_inputs, to_device, to_numpy
    from paper_2506_15976_amd.inputs import make_inputs
    for dtype, (B, D, L) in (("fp32", (2, 9, 1500)), ("bf16", (1, 12, 2050)), ("fp32", (1, 5, 100))):
        sf = make_inputs(B, D, 16, L, seed=7700 + L, dtype=dtype, random_A=True)
        sb = make_inputs(B, D, 16, L, seed=7701 + L, dtype=dtype, random_A=True)
        sb["z"] = sf["z"]
        df, db = to_device(sf, dtype), to_device(sb, dtype)
        got = lb.lbscan_bidir_fwd(fwd_inputs(df), fwd_inputs(db))
        torch.cuda.synchronize()
        assert_close(to_numpy(got), oracle.bidir_fwd(fwd_inputs(sf), fwd_inputs(sb)), dtype, "bidir")
        got = lb.lbscan_fwd(**fwd_inputs(df), window=5)
        torch.cuda.synchronize()
        assert_close(to_numpy(got), oracle.fwd(**fwd_inputs(sf), window=5), dtype, "window 5")


def test_matches_row_per_lane_kernels_at_full_size(lb, oracle):
    """The 4096-token workload in the launch the library picks by itself (this kernel)
    against the oracle, and against the row-per-lane path forced on the same inputs."""
    import torch
    from gpu_util import assert_close, fwd_inputs, to_device, to_numpy
    from paper_2506_15976_amd.inputs import WORKLOADS, make_workload
    w = WORKLOADS["hires_4096"]
    s = make_workload("hires_4096")
    dev = to_device(s, w["dtype"])
    got = lb.lbscan_fwd(**fwd_inputs(dev), window=w["window"])
    lb.lbscan_set_option("mapping", 1)
    try:
        other = lb.lbscan_fwd(**fwd_inputs(dev), window=w["window"])
    finally:
        lb.lbscan_set_option("mapping", 0)
    torch.cuda.synchronize()
    ref = oracle.fwd(**fwd_inputs(s), window=w["window"])
    assert_close(to_numpy(got), ref, w["dtype"], "chunk per lane")
    assert_close(to_numpy(other), ref, w["dtype"], "row per lane")
