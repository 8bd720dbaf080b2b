"""Pins for the oracle's state-in / state-out entry points (no GPU).

Algorithm 1 of the paper starts the forward state at zero.  Processing a long
sequence in chunks needs the state to enter and leave a call; what that must
compute is fixed by Eq. 1 alone, so it is pinned against

  * the unrolled sum of Eq. 1 with the entering state decayed by the product of
    abar (closed form, written out here),
  * the chunk identity: one call over the row equals two calls over its halves
    with the state handed over, when the cut is a multiple of the window,
  * central differences for the gradient w.r.t. the entering state and for every
    gradient when the loss also depends on the leaving state,
  * the chain rule across the cut (gradients of the two chunk calls add up to
    those of the single call).
"""
import math

import numpy as np
import pytest

from test_oracle_pins import _GRAD_OF, _brute_force, _rand_problem, _timestep


def _state(B, D, N, seed):
    return np.random.default_rng(seed).standard_normal((B, D, N))


@pytest.mark.parametrize("L,M", [(13, 4), (9, 3), (8, 1), (6, 9)])
def test_entering_state_matches_unrolled_sums(oracle, L, M):
    """out(h0) = out(0) + gate * sum_n C_t exp(A sum_{r<=t} dt_r) h0 and
    hT = exp(A sum_r dt_r) h0 + sum_s exp(A sum_{r>s} dt_r) u_s."""
    p = _rand_problem(2, 3, 3, L, seed=1200 + L)
    h0 = _state(2, 3, 3, 1201 + L)
    out, hT = oracle.fwd(**p, window=M, delta_softplus=True, h0=h0, return_state=True)
    dt = _timestep(p, True)
    want = _brute_force(p, M, True)
    want_hT = np.zeros_like(h0)
    for b in range(2):
        for d in range(3):
            for n in range(3):
                a = p["A"][d, n]
                for t in range(L):
                    extra = p["Cm"][b, n, t] * math.exp(a * dt[b, d, : t + 1].sum()) * h0[b, d, n]
                    zz = p["z"][b, d, t]
                    want[b, d, t] += extra * zz / (1.0 + math.exp(-zz))
                acc = math.exp(a * dt[b, d].sum()) * h0[b, d, n]
                for s in range(L):
                    acc += math.exp(a * dt[b, d, s + 1:].sum()) * dt[b, d, s] * p["Bm"][b, n, s] * p["x"][b, d, s]
                want_hT[b, d, n] = acc
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(hT, want_hT, rtol=1e-11, atol=1e-12)


def test_zero_entering_state_is_the_plain_call(oracle):
    p = _rand_problem(1, 2, 3, 10, seed=1210)
    base = oracle.fwd(**p, window=4, delta_softplus=True)
    out, _ = oracle.fwd(**p, window=4, delta_softplus=True, h0=np.zeros((1, 2, 3)), return_state=True)
    np.testing.assert_array_equal(out, base)


def _cut(p, lo, hi):
    q = dict(p)
    for k in ("x", "delta", "Bm", "Cm", "z"):
        if p[k] is not None:
            q[k] = np.ascontiguousarray(p[k][..., lo:hi])
    return q


@pytest.mark.parametrize("L,M,cut", [(23, 4, 8), (23, 4, 20), (17, 3, 9), (12, 1, 5), (16, 8, 8)])
def test_two_chunks_equal_one_call(oracle, L, M, cut):
    p = _rand_problem(2, 3, 4, L, seed=1220 + L)
    h0 = _state(2, 3, 4, 1221)
    whole, hT = oracle.fwd(**p, window=M, delta_softplus=True, h0=h0, return_state=True)
    o1, h1 = oracle.fwd(**_cut(p, 0, cut), window=M, delta_softplus=True, h0=h0, return_state=True)
    o2, h2 = oracle.fwd(**_cut(p, cut, L), window=M, delta_softplus=True, h0=h1, return_state=True)
    np.testing.assert_allclose(np.concatenate([o1, o2], axis=-1), whole, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(h2, hT, rtol=1e-12, atol=1e-13)


def test_cut_inside_a_window_changes_the_result(oracle):
    """The local backward state does not cross calls: a cut that is not a
    multiple of the window is a different operator (guards the test above)."""
    p = _rand_problem(1, 2, 2, 12, seed=1230)
    whole = oracle.fwd(**p, window=4, delta_softplus=True)
    o1, h1 = oracle.fwd(**_cut(p, 0, 6), window=4, delta_softplus=True, return_state=True)
    o2 = oracle.fwd(**_cut(p, 6, 12), window=4, delta_softplus=True, h0=h1)
    assert np.max(np.abs(np.concatenate([o1, o2], axis=-1) - whole)) > 1e-3


@pytest.mark.parametrize("L,M,softplus", [(13, 4, True), (9, 3, False), (8, 1, True), (5, 7, True)])
def test_state_gradients_match_central_differences(oracle, L, M, softplus):
    p = _rand_problem(2, 2, 3, L, softplus=softplus, seed=1240 + L)
    r = np.random.default_rng(1241 + L)
    h0 = r.standard_normal((2, 2, 3))
    dout = r.standard_normal(p["x"].shape)
    dhT = r.standard_normal(h0.shape)
    g = oracle.bwd(**p, dout=dout, window=M, delta_softplus=softplus, h0=h0, dhT=dhT)

    def loss(q, hh):
        out, hT = oracle.fwd(**q, window=M, delta_softplus=softplus, h0=hh, return_state=True)
        return float(np.sum(dout * out) + np.sum(dhT * hT))

    h = 1e-6
    names = dict(_GRAD_OF, h0="dh0")
    for name, gname in names.items():
        arr = h0 if name == "h0" else p[name]
        flat_idx = r.choice(arr.size, size=min(arr.size, 10), replace=False)
        scale = np.sqrt(np.mean(g[gname] ** 2)) + 1e-30
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += h
            lo[idx] -= h
            if name == "h0":
                fd = (loss(p, hi) - loss(p, lo)) / (2 * h)
            else:
                fd = (loss(dict(p, **{name: hi}), h0) - loss(dict(p, **{name: lo}), h0)) / (2 * h)
            assert abs(fd - g[gname][idx]) <= 2e-6 * max(abs(fd), scale), (name, idx, fd, g[gname][idx])


def test_gradients_chain_across_the_cut(oracle):
    L, M, cut = 20, 4, 12
    p = _rand_problem(2, 3, 3, L, seed=1250)
    r = np.random.default_rng(1251)
    h0 = r.standard_normal((2, 3, 3))
    dout = r.standard_normal(p["x"].shape)
    dhT = r.standard_normal(h0.shape)
    whole = oracle.bwd(**p, dout=dout, window=M, delta_softplus=True, h0=h0, dhT=dhT)
    p1, p2 = _cut(p, 0, cut), _cut(p, cut, L)
    _, h1 = oracle.fwd(**p1, window=M, delta_softplus=True, h0=h0, return_state=True)
    g2 = oracle.bwd(**p2, dout=np.ascontiguousarray(dout[..., cut:]), window=M, delta_softplus=True,
                    h0=h1, dhT=dhT)
    g1 = oracle.bwd(**p1, dout=np.ascontiguousarray(dout[..., :cut]), window=M, delta_softplus=True,
                    h0=h0, dhT=g2["dh0"])
    for k in ("dx", "ddelta", "dz", "dBm", "dCm"):
        np.testing.assert_allclose(np.concatenate([g1[k], g2[k]], axis=-1), whole[k], rtol=1e-11, atol=1e-12)
    for k in ("dA", "dDskip", "ddelta_bias"):
        np.testing.assert_allclose(g1[k] + g2[k], whole[k], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g1["dh0"], whole["dh0"], rtol=1e-11, atol=1e-12)


def test_plain_backward_is_the_state_backward_with_nothing_passed(oracle):
    p = _rand_problem(1, 2, 2, 9, seed=1260)
    dout = np.random.default_rng(1261).standard_normal(p["x"].shape)
    a = oracle.bwd(**p, dout=dout, window=4, delta_softplus=True)
    b = oracle.bwd(**p, dout=dout, window=4, delta_softplus=True, h0=np.zeros((1, 2, 2)))
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_empty_row_passes_the_state_through(oracle):
    p = _rand_problem(1, 2, 3, 0, seed=1270)
    h0 = _state(1, 2, 3, 1271)
    out, hT = oracle.fwd(**p, window=4, delta_softplus=True, h0=h0, return_state=True)
    assert out.shape == (1, 2, 0)
    np.testing.assert_array_equal(hT, h0)
