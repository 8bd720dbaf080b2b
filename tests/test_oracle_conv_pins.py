"""Pins for the oracle of the block's pre-scan step (depthwise causal convolution
along the sequence, then SiLU; Algorithm 1 of arXiv 2506.15976 names it without
detail).  Pinned against a library FIR filter, sums written out by hand, the flip
identity for the reversed direction and central differences."""
import math

import numpy as np
import pytest
import scipy.signal


def _problem(B, D, L, K, seed, bias=True):
    r = np.random.default_rng(seed)
    return dict(x=r.standard_normal((B, D, L)), weight=r.standard_normal((D, K)),
                bias=r.standard_normal(D) if bias else None)


@pytest.mark.parametrize("L,K", [(17, 4), (5, 4), (3, 4), (9, 1), (12, 2), (1, 3)])
def test_matches_library_fir_filter(oracle, L, K):
    p = _problem(2, 3, L, K, 300 + L + K)
    y = oracle.conv1d_fwd(**p, activation=False)
    for b in range(2):
        for d in range(3):
            # tap k multiplies x[t-(K-1)+k]: the FIR coefficients are the taps reversed
            want = scipy.signal.lfilter(p["weight"][d, ::-1], [1.0], p["x"][b, d]) + p["bias"][d]
            np.testing.assert_allclose(y[b, d], want, rtol=1e-12, atol=1e-13)


def test_activation_and_hand_written_sum(oracle):
    p = _problem(1, 2, 6, 4, 310)
    y = oracle.conv1d_fwd(**p)
    x, w, bias = p["x"][0, 1], p["weight"][1], p["bias"][1]
    # output 4 sees inputs 1..4, output 1 sees inputs (-2, -1 -> zero), 0, 1
    pre4 = bias + w[0] * x[1] + w[1] * x[2] + w[2] * x[3] + w[3] * x[4]
    pre1 = bias + w[2] * x[0] + w[3] * x[1]
    assert y[0, 1, 4] == pytest.approx(pre4 / (1 + math.exp(-pre4)), rel=1e-13)
    assert y[0, 1, 1] == pytest.approx(pre1 / (1 + math.exp(-pre1)), rel=1e-13)


def test_reverse_is_the_operator_on_the_flipped_sequence(oracle):
    p = _problem(2, 3, 11, 4, 320)
    rev = oracle.conv1d_fwd(**p, reverse=True)
    flipped = oracle.conv1d_fwd(**dict(p, x=np.ascontiguousarray(p["x"][..., ::-1])))
    np.testing.assert_allclose(rev, flipped[..., ::-1], rtol=1e-13, atol=1e-15)
    # output 0 of the reversed operator sees inputs 0..K-1 with the taps mirrored
    x, w = p["x"][1, 2], p["weight"][2]
    pre = p["bias"][2] + sum(w[3 - j] * x[j] for j in range(4))
    assert rev[1, 2, 0] == pytest.approx(pre / (1 + math.exp(-pre)), rel=1e-13)


def test_without_bias(oracle):
    p = _problem(1, 2, 7, 3, 330, bias=False)
    y = oracle.conv1d_fwd(**p, activation=False)
    want = scipy.signal.lfilter(p["weight"][0, ::-1], [1.0], p["x"][0, 0])
    np.testing.assert_allclose(y[0, 0], want, rtol=1e-12, atol=1e-13)
    g = oracle.conv1d_bwd(**p, dy=np.ones_like(p["x"]), activation=False)
    assert g["dbias"] is None


@pytest.mark.parametrize("L,K,activation,reverse", [(13, 4, True, False), (6, 4, True, True),
                                                    (9, 2, False, False), (3, 4, True, False)])
def test_gradients_match_central_differences(oracle, L, K, activation, reverse):
    p = _problem(2, 3, L, K, 340 + L)
    dy = np.random.default_rng(341 + L).standard_normal(p["x"].shape)
    g = oracle.conv1d_bwd(**p, dy=dy, activation=activation, reverse=reverse)
    loss = lambda q: float(np.sum(dy * oracle.conv1d_fwd(**q, activation=activation, reverse=reverse)))
    h = 1e-6
    for name, gname in (("x", "dx"), ("weight", "dweight"), ("bias", "dbias")):
        arr = p[name]
        scale = np.sqrt(np.mean(g[gname] ** 2)) + 1e-30
        for fi in range(0, arr.size, max(1, arr.size // 15)):
            idx = np.unravel_index(fi, arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += h
            lo[idx] -= h
            fd = (loss(dict(p, **{name: hi})) - loss(dict(p, **{name: lo}))) / (2 * h)
            assert abs(fd - g[gname][idx]) <= 2e-6 * max(abs(fd), scale), (name, idx, fd, g[gname][idx])


def test_adjoint_identity_without_activation(oracle):
    """Linear in x without activation and bias: <dy, J v> = <J^T dy, v>."""
    p = _problem(2, 3, 14, 4, 350, bias=False)
    r = np.random.default_rng(351)
    v, dy = r.standard_normal(p["x"].shape), r.standard_normal(p["x"].shape)
    Jv = oracle.conv1d_fwd(**dict(p, x=v), activation=False)
    g = oracle.conv1d_bwd(**p, dy=dy, activation=False)
    assert float(np.sum(dy * Jv)) == pytest.approx(float(np.sum(g["dx"] * v)), rel=1e-12)


def test_empty(oracle):
    p = _problem(1, 2, 0, 4, 360)
    assert oracle.conv1d_fwd(**p).shape == (1, 2, 0)
    g = oracle.conv1d_bwd(**p, dy=np.empty((1, 2, 0)))
    assert np.all(g["dweight"] == 0) and np.all(g["dbias"] == 0)
