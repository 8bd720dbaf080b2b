"""Randomised pins for the oracle (hypothesis): for arbitrary small shapes, window
lengths and optional inputs the oracle equals the unrolled sums of Eq. 1 / 7 / 8, its
gradient satisfies the adjoint identity, and reversing time maps windows anchored
at the start onto windows anchored at the end."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from test_oracle_pins import _brute_force, _rand_problem

shapes = st.tuples(st.integers(1, 2), st.integers(1, 3), st.integers(1, 3), st.integers(1, 12))


@settings(max_examples=40, deadline=None)
@given(shape=shapes, M=st.integers(1, 14), seed=st.integers(0, 10_000), softplus=st.booleans(),
       gate=st.booleans(), skip=st.booleans(), bias=st.booleans())
def test_forward_equals_unrolled_sums(oracle, shape, M, seed, softplus, gate, skip, bias):
    B, D, N, L = shape
    p = _rand_problem(B, D, N, L, softplus=softplus, gate=gate, skip=skip, bias=bias, seed=seed)
    got = oracle.fwd(**p, window=M, delta_softplus=softplus)
    np.testing.assert_allclose(got, _brute_force(p, M, softplus), rtol=1e-11, atol=1e-12)


@settings(max_examples=40, deadline=None)
@given(shape=shapes, M=st.integers(1, 14), seed=st.integers(0, 10_000))
def test_backward_is_the_adjoint_of_the_forward_in_x(oracle, shape, M, seed):
    """Without a gate out is linear in x: <dout, J v> = <J^T dout, v>."""
    B, D, N, L = shape
    p = _rand_problem(B, D, N, L, gate=False, seed=seed)
    r = np.random.default_rng(seed + 1)
    v, dout = r.standard_normal(p["x"].shape), r.standard_normal(p["x"].shape)
    Jv = oracle.fwd(**dict(p, x=v), window=M, delta_softplus=True)
    g = oracle.bwd(**p, dout=dout, window=M, delta_softplus=True)
    assert float(np.sum(dout * Jv)) == pytest.approx(float(np.sum(g["dx"] * v)), rel=1e-10, abs=1e-12)


@settings(max_examples=30, deadline=None)
@given(shape=shapes, k=st.integers(1, 4), M=st.integers(1, 5), seed=st.integers(0, 10_000))
def test_whole_windows_commute_with_time_reversal_of_the_local_part(oracle, shape, k, M, seed):
    """With L a multiple of M the windows of the reversed sequence are the reversed
    windows, so (local part of the scan) = (plain scan of the reversed sequence,
    restarted at every window, minus its own input term): checked through
    out(M) - out(1) on the original against the same difference built from
    per-window plain scans of the flipped windows."""
    B, D, N, _ = shape
    L = k * M
    p = _rand_problem(B, D, N, L, gate=False, skip=False, seed=seed)
    local = oracle.fwd(**p, window=M, delta_softplus=True) - oracle.fwd(**p, window=1, delta_softplus=True)
    want = np.zeros_like(local)
    for w0 in range(0, L, M):
        q = {key: (np.ascontiguousarray(val[..., w0:w0 + M][..., ::-1]) if isinstance(val, np.ndarray) and val.ndim == 3
                   else val) for key, val in p.items()}
        plain = oracle.fwd(**q, window=1, delta_softplus=True)            # sum_n C h, h inclusive
        # subtract the step's own input term sum_n C u
        dt = np.log1p(np.exp(q["delta"] + q["delta_bias"][None, :, None]))
        own = np.einsum("bnl,bdl->bdl", q["Cm"] * q["Bm"], dt * q["x"])
        want[..., w0:w0 + M] = (plain - own)[..., ::-1]
    np.testing.assert_allclose(local, want, rtol=1e-10, atol=1e-12)
