"""The entry points enqueue kernels only (no allocation, no synchronisation, no
memset node), so a call can be recorded into a HIP graph.  Every replay is checked
against the eager result, with eager work and synchronisations between replays."""
import ctypes

import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lb():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2506_15976_amd as pkg
    pkg.load()
    return pkg


def _stream_ptr(stream):
    return ctypes.c_void_p(stream.cuda_stream)


def _workspace(lb, args, which, device):
    import torch
    need = lb.lbscan_workspace_bytes(args, which)
    ws = torch.empty(max(need // 4, 1), dtype=torch.float32, device=device)
    args.workspace = ws.data_ptr()
    args.workspace_bytes = ws.numel() * 4
    return ws


@pytest.mark.parametrize("shape,window,segments,mapping", [
    ((2, 70, 16, 197), 4, 0, 0), ((1, 64, 16, 900), 8, 3, 0), ((2, 64, 16, 100), 5, 0, 0),
    ((2, 9, 16, 2500), 8, 0, 2),        # the chunk-per-lane kernel
])
def test_forward_call_replays_from_a_graph(lb, shape, window, segments, mapping):
    import torch
    from gpu_util import fwd_inputs, to_device
    from paper_2506_15976_amd.inputs import make_inputs
    B, D, N, L = shape
    lib = lb.load()
    lb.lbscan_set_option("segments", segments)
    lb.lbscan_set_option("mapping", mapping)
    try:
        dev = fwd_inputs(to_device(make_inputs(B, D, N, L, seed=8100 + L), "fp32"))
        y_eager = lb.lbscan_fwd(**dev, window=window)
        y = torch.zeros_like(y_eager)
        a = lb.make_args(**dev, window=window, y=y)
        ws = _workspace(lb, a, 0, y.device)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                rc = lib.lbscan_fwd(ctypes.byref(a), _stream_ptr(torch.cuda.current_stream()))
        assert rc == 0
        for k in range(3):
            y.fill_(float("nan"))
            ws.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, y_eager), f"replay {k}"
            # eager work of the program's own between the replays
            again = lb.lbscan_fwd(**dev, window=window)
            torch.cuda.synchronize()
            assert torch.equal(again, y_eager)
    finally:
        lb.lbscan_set_option("segments", 0)
        lb.lbscan_set_option("mapping", 0)


def test_backward_call_replays_from_a_graph(lb, oracle):
    import torch
    from gpu_util import assert_close, fwd_inputs, to_device, to_numpy
    from paper_2506_15976_amd.inputs import make_inputs
    lib = lb.load()
    s = make_inputs(2, 70, 16, 120, seed=8200, with_dout=True)
    dev = to_device(s, "fp32")
    f = fwd_inputs(dev)
    ref = oracle.bwd(**fwd_inputs(s), dout=s["dout"], window=4)
    a = lb.make_args(**f, window=4)
    ws = _workspace(lb, a, 1, dev["x"].device)
    g = {k: torch.empty_like(dev["x"]) for k in ("dx", "ddelta", "dz")}
    g.update(dBm=torch.empty_like(dev["Bm"]), dCm=torch.empty_like(dev["Cm"]), dA=torch.empty_like(dev["A"]),
             dDskip=torch.empty_like(dev["Dskip"]), ddelta_bias=torch.empty_like(dev["delta_bias"]))
    order = ("dx", "ddelta", "dz", "dBm", "dCm", "dA", "dDskip", "ddelta_bias")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            rc = lib.lbscan_bwd(ctypes.byref(a), ctypes.c_void_p(dev["dout"].data_ptr()),
                                *[ctypes.c_void_p(g[k].data_ptr()) for k in order],
                                _stream_ptr(torch.cuda.current_stream()))
    assert rc == 0
    for k in range(3):
        for t in g.values():
            t.fill_(float("nan"))          # the call must overwrite, also its accumulators
        ws.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in order:
            assert_close(to_numpy(g[name]), ref[name], "fp32", f"{name} (replay {k})")
        lb.lbscan_fwd(**f, window=4)       # eager work between the replays
        torch.cuda.synchronize()


def test_forward_is_bit_reproducible(lb):
    """The forward pass has no atomics: two runs give the same bits."""
    import torch
    from gpu_util import fwd_inputs, to_device
    from paper_2506_15976_amd.inputs import make_inputs
    for shape, window in (((2, 130, 16, 197), 4), ((1, 64, 16, 3000), 8), ((2, 64, 16, 77), 7)):
        dev = fwd_inputs(to_device(make_inputs(*shape, seed=8300), "fp32"))
        a = lb.lbscan_fwd(**dev, window=window)
        b = lb.lbscan_fwd(**dev, window=window)
        torch.cuda.synchronize()
        assert torch.equal(a, b)


def test_backward_of_an_empty_row_zeroes_the_channel_sums(lb):
    import torch
    x = torch.empty((2, 8, 0), device="cuda")
    Bm = torch.empty((2, 4, 0), device="cuda")
    A = -torch.ones((8, 4), device="cuda")
    Dk = torch.ones(8, device="cuda")
    g = lb.lbscan_bwd(x, x, A, Bm, Bm, Dk, dout=x, window=4)
    torch.cuda.synchronize()
    assert g["dx"].shape == (2, 8, 0)
    assert torch.count_nonzero(g["dA"]) == 0 and torch.count_nonzero(g["dDskip"]) == 0
