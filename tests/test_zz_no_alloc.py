"""The allocation-free forward entry point (scratch in a fixed device array) against
lbscan_fwd, through the C ABI: two calls in a row, the second with a smaller input."""
import ctypes

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


def _both(lb, oracle, shape, window, dtype="fp32", reverse=False, check_oracle=True):
    """out of lbscan_fwd (caller's workspace) and of lbscan_fwd_static on the same
    inputs; the two run the same kernels, so they must agree bit for bit."""
    import torch
    from gpu_util import assert_close, flip_time, fwd_inputs, to_device, to_numpy
    from paper_2506_15976_amd import binding
    from paper_2506_15976_amd.inputs import make_inputs
    B, D, N, L = shape
    s = make_inputs(B, D, N, L, seed=4200 + L, dtype=dtype)
    dev = to_device(s, dtype)
    lib = lb.load()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    y_ref = torch.empty_like(dev["x"])
    a = lb.make_args(**fwd_inputs(dev), window=window, reverse=reverse, y=y_ref)
    need = lb.lbscan_workspace_bytes(a, binding.WS_FWD)
    ws = torch.empty(max(need // 4, 1), dtype=torch.float32, device="cuda:0")
    a.workspace, a.workspace_bytes = ws.data_ptr(), need
    assert lib.lbscan_fwd(ctypes.byref(a), stream) == 0

    y_new = torch.full_like(dev["x"], float("nan"))
    b = lb.make_args(**fwd_inputs(dev), window=window, reverse=reverse, y=y_new)     # no workspace at all
    assert b.workspace is None or b.workspace == 0
    before = torch.cuda.memory_allocated()
    rc = lib.lbscan_fwd_static(ctypes.byref(b), stream)
    assert rc == 0, lib.lbscan_last_error()
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    got, ref = to_numpy(y_new), to_numpy(y_ref)
    assert np.array_equal(got, ref), f"max diff {np.max(np.abs(got - ref))}"
    if check_oracle:
        src = flip_time(s) if reverse else s
        want = oracle.fwd(**fwd_inputs(src), window=window)
        assert_close(got, want[..., ::-1] if reverse else want, dtype)
    return need


def test_static_scratch_two_calls_second_smaller(lb, oracle):
    # long rows, few channels: rows are cut into segments and the carried states go
    # through the scratch array
    n1 = _both(lb, oracle, (1, 130, 16, 6000), 4)
    n2 = _both(lb, oracle, (1, 64, 16, 2500), 4, reverse=True)
    assert n1 > n2 > 0
    # again the larger one: what the smaller call left behind does not matter
    _both(lb, oracle, (1, 130, 16, 6000), 4, check_oracle=False)
    # sizes that need no scratch, and a window length that takes the two-pass path
    assert _both(lb, oracle, (16, 1024, 16, 40), 4) == 0
    assert _both(lb, oracle, (1, 64, 16, 3000), 8, dtype="bf16") > 0
    _both(lb, oracle, (1, 64, 16, 2000), 3)


def test_static_scratch_rejects_sizes_beyond_the_array(lb):
    import torch
    from gpu_util import fwd_inputs, to_device
    from paper_2506_15976_amd import binding
    from paper_2506_15976_amd.inputs import make_inputs
    # bf16 storage with a window length that needs the fp32 first-pass buffer: B*D*L*4 bytes
    s = make_inputs(1, 1024, 16, 4096, seed=1, dtype="bf16")
    dev = to_device(s, "bf16")
    y = torch.empty_like(dev["x"])
    a = lb.make_args(**fwd_inputs(dev), window=3, y=y)
    need = lb.lbscan_workspace_bytes(a, binding.WS_FWD)
    assert need > binding.STATIC_SCRATCH_BYTES
    lib = lb.load()
    rc = lib.lbscan_fwd_static(ctypes.byref(a), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == binding.EWORKSPACE
    msg = lib.lbscan_last_error().decode()
    assert str(need) in msg and str(binding.STATIC_SCRATCH_BYTES) in msg
    with pytest.raises(lb.LbscanError) as ei:
        lb.lbscan_fwd_static(**fwd_inputs(dev), out=y, window=3)
    assert ei.value.code == binding.EWORKSPACE
