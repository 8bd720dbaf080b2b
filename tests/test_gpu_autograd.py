"""The autograd wiring (paper_2506_15976_amd.autograd) returns the library's
gradients for a scalar loss, checked against the fp64 oracle."""
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


@pytest.mark.parametrize("reverse", [False, True])
def test_scan_gradients_through_autograd(lb, oracle, reverse):
    import torch
    from gpu_util import assert_close, flip_time, fwd_inputs, to_device, to_numpy
    from paper_2506_15976_amd.autograd import lb_selective_scan
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(2, 70, 16, 90, seed=9300, with_dout=True, random_A=True)
    r = np.random.default_rng(9301)
    h0 = r.standard_normal((2, 70, 16)).astype(np.float32)
    dhT = r.standard_normal((2, 70, 16)).astype(np.float32)
    dev = fwd_inputs(to_device(s, "fp32"))
    leaves = {k: v.clone().requires_grad_(True) for k, v in dev.items()}
    h0d = torch.from_numpy(h0).cuda().requires_grad_(True)
    out, hT = lb_selective_scan(**leaves, window=4, reverse=reverse, h0=h0d, return_state=True)
    dout = torch.from_numpy(s["dout"]).cuda()
    loss = (out * dout).sum() + (hT * torch.from_numpy(dhT).cuda()).sum()
    loss.backward()
    torch.cuda.synchronize()
    src = flip_time(s) if reverse else s
    ref = oracle.bwd(**fwd_inputs(src), dout=src["dout"], window=4, h0=h0, dhT=dhT)
    names = dict(x="dx", delta="ddelta", z="dz", Bm="dBm", Cm="dCm", A="dA", Dskip="dDskip",
                 delta_bias="ddelta_bias")
    for k, gk in names.items():
        want = ref[gk][..., ::-1] if reverse and ref[gk].ndim == 3 else ref[gk]
        assert_close(to_numpy(leaves[k].grad), want, "fp32", gk)
    assert_close(to_numpy(h0d.grad), ref["dh0"], "fp32", "dh0")


def test_scan_without_optionals_and_state(lb, oracle):
    import torch
    from gpu_util import assert_close, to_device, to_numpy
    from paper_2506_15976_amd.autograd import lb_selective_scan
    from paper_2506_15976_amd.inputs import make_inputs
    s = make_inputs(1, 64, 16, 50, seed=9310, with_dout=True, with_z=False)
    dev = to_device(s, "fp32")
    x = dev["x"].clone().requires_grad_(True)
    A = dev["A"].clone().requires_grad_(True)
    out = lb_selective_scan(x, dev["delta"], A, dev["Bm"], dev["Cm"], window=8)
    (out * dev["dout"]).sum().backward()
    torch.cuda.synchronize()
    ref = oracle.bwd(s["x"], s["delta"], s["A"], s["Bm"], s["Cm"], dout=s["dout"], window=8)
    assert_close(to_numpy(x.grad), ref["dx"], "fp32", "dx")
    assert_close(to_numpy(A.grad), ref["dA"], "fp32", "dA")


def test_conv_gradients_through_autograd(lb, oracle):
    import torch
    from gpu_util import assert_close, to_numpy
    from paper_2506_15976_amd.autograd import causal_conv1d_silu
    r = np.random.default_rng(9320)
    x = r.standard_normal((2, 6, 130)).astype(np.float32)
    w = (0.5 * r.standard_normal((6, 4))).astype(np.float32)
    b = r.standard_normal(6).astype(np.float32)
    dy = r.standard_normal(x.shape).astype(np.float32)
    xd, wd, bd = (torch.from_numpy(a).cuda().requires_grad_(True) for a in (x, w, b))
    y = causal_conv1d_silu(xd, wd, bd)
    (y * torch.from_numpy(dy).cuda()).sum().backward()
    torch.cuda.synchronize()
    ref = oracle.conv1d_bwd(x, w, b, dy=dy)
    assert_close(to_numpy(xd.grad), ref["dx"], "fp32", "dx")
    assert_close(to_numpy(wd.grad), ref["dweight"], "fp32", "dweight")
    assert_close(to_numpy(bd.grad), ref["dbias"], "fp32", "dbias")
