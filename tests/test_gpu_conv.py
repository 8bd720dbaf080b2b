"""GPU parity of lbscan_conv1d_fwd / lbscan_conv1d_bwd (the block's pre-scan step)
against the fp64 CPU oracle, element by element, through the C ABI."""
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


def _inputs(B, D, L, K, seed, dtype="fp32", bias=True):
    from paper_2506_15976_amd.inputs import round_to_bf16
    r = np.random.default_rng(seed)
    x = r.standard_normal((B, D, L)).astype(np.float32)
    dy = r.standard_normal((B, D, L)).astype(np.float32)
    if dtype == "bf16":
        x, dy = round_to_bf16(x), round_to_bf16(dy)
    w = (r.standard_normal((D, K)) / np.sqrt(K)).astype(np.float32)
    b = r.standard_normal(D).astype(np.float32) if bias else None
    return dict(x=x, weight=w, bias=b, dy=dy)


def _dev(s, dtype):
    from gpu_util import to_device
    d = to_device({"x": s["x"], "dout": s["dy"]}, dtype)
    import torch
    out = dict(x=d["x"], dy=d["dout"], weight=torch.from_numpy(s["weight"]).cuda(),
               bias=None if s["bias"] is None else torch.from_numpy(s["bias"]).cuda())
    return out


def _check(lb, oracle, s, *, dtype="fp32", activation=True, reverse=False):
    import torch
    from gpu_util import assert_close, to_numpy
    d = _dev(s, dtype)
    y = lb.lbscan_conv1d_fwd(d["x"], d["weight"], d["bias"], activation=activation, reverse=reverse)
    g = lb.lbscan_conv1d_bwd(d["x"], d["weight"], d["bias"], dy=d["dy"], activation=activation, reverse=reverse)
    torch.cuda.synchronize()
    ref = oracle.conv1d_fwd(s["x"], s["weight"], s["bias"], activation=activation, reverse=reverse)
    rg = oracle.conv1d_bwd(s["x"], s["weight"], s["bias"], dy=s["dy"], activation=activation, reverse=reverse)
    assert_close(to_numpy(y), ref, dtype, "y")
    assert_close(to_numpy(g["dx"]), rg["dx"], dtype, "dx")
    assert_close(to_numpy(g["dweight"]), rg["dweight"], "fp32", "dweight")
    if s["bias"] is None:
        assert g["dbias"] is None
    else:
        assert_close(to_numpy(g["dbias"]), rg["dbias"], "fp32", "dbias")


@pytest.mark.parametrize("shape", [
    # (B, D, L): ragged tails, one partial chunk, several chunks, chunk edges at 252 / 256 tokens
    (2, 5, 197), (1, 3, 1), (2, 4, 3), (1, 2, 4), (3, 7, 255), (1, 2, 256), (1, 2, 257), (2, 3, 252),
    (1, 2, 253), (1, 4, 1000), (1, 1, 4096), (2, 3, 509),
])
@pytest.mark.parametrize("reverse", [False, True])
def test_shapes_width_four(lb, oracle, shape, reverse):
    B, D, L = shape
    _check(lb, oracle, _inputs(B, D, L, 4, 6100 + L), reverse=reverse)


@pytest.mark.parametrize("K", [1, 2, 3])
@pytest.mark.parametrize("reverse", [False, True])
def test_other_widths(lb, oracle, K, reverse):
    _check(lb, oracle, _inputs(2, 6, 301, K, 6200 + K), reverse=reverse)


def test_without_bias_and_without_activation(lb, oracle):
    _check(lb, oracle, _inputs(2, 6, 130, 4, 6300, bias=False))
    _check(lb, oracle, _inputs(2, 6, 130, 4, 6301), activation=False)


@pytest.mark.parametrize("L", [96, 197, 5, 7, 261, 1025])   # odd row length: rows start at odd bf16 elements
def test_bf16_storage(lb, oracle, L):
    _check(lb, oracle, _inputs(2, 8, L, 4, 6400 + L, dtype="bf16"), dtype="bf16")
    _check(lb, oracle, _inputs(2, 8, L, 4, 6401 + L, dtype="bf16"), dtype="bf16", reverse=True)


def test_vim_small_shape(lb, oracle):
    """The (B, D, L) of the vim_small workload, as the benchmark would run it."""
    _check(lb, oracle, _inputs(128, 768, 197, 4, 6500))


def test_unsupported_width_and_empty(lb):
    import torch
    x = torch.zeros((1, 2, 8), device="cuda")
    w = torch.zeros((2, 5), device="cuda")
    with pytest.raises(lb.LbscanError) as ei:
        lb.lbscan_conv1d_fwd(x, w)
    assert ei.value.code == -2
    x0 = torch.zeros((1, 2, 0), device="cuda")
    w4 = torch.ones((2, 4), device="cuda")
    b = torch.ones(2, device="cuda")
    assert lb.lbscan_conv1d_fwd(x0, w4, b).shape == (1, 2, 0)
    g = lb.lbscan_conv1d_bwd(x0, w4, b, dy=x0)
    torch.cuda.synchronize()
    assert torch.count_nonzero(g["dweight"]) == 0 and torch.count_nonzero(g["dbias"]) == 0
