"""Pins for the fp64 CPU oracle (no GPU).

The paper (arXiv 2506.15976) prints no worked numerical example for the scan:
its figures use symbolic states only.  So the oracle is pinned against what the
definitions and the mathematics fix instead:

  * unrolled O(L^2) sums written straight from Eq. 1, Eq. 7 and Eq. 8,
  * a library IIR filter for the constant-coefficient special case of Eq. 1,
  * closed forms (geometric sums), impulse responses, window locality,
  * the relation between the local scan with one window and the global
    bi-directional scan of Eq. 4-6,
  * central finite differences and an adjoint identity for every gradient.

Each check is chosen so that a dropped term, a wrong sign, an off-by-one in the
window boundaries or a transposed operand fails at least one of them.
"""
import math

import numpy as np
import pytest
import scipy.signal

RNG = np.random.default_rng(7)


def _rand_problem(B, D, N, L, *, softplus=True, gate=True, skip=True, bias=True, seed=0):
    r = np.random.default_rng(seed)
    p = dict(
        x=r.standard_normal((B, D, L)),
        delta=0.5 * r.standard_normal((B, D, L)) + (0.0 if softplus else 1.0),
        A=-r.uniform(0.3, 3.0, size=(D, N)),
        Bm=r.standard_normal((B, N, L)),
        Cm=r.standard_normal((B, N, L)),
        Dskip=r.standard_normal(D) if skip else None,
        z=r.standard_normal((B, D, L)) if gate else None,
        delta_bias=r.uniform(-2.0, 0.5, size=D) if bias else None,
    )
    if not softplus:
        # keep the time step positive without softplus, so abar stays below one
        p["delta"] = np.abs(p["delta"]) * 0.3 + 0.01
        if bias:
            p["delta_bias"] = r.uniform(0.0, 0.2, size=D)
    return p


def _timestep(p, softplus):
    v = p["delta"] + (p["delta_bias"][None, :, None] if p["delta_bias"] is not None else 0.0)
    return np.where(v > 20, v, np.log1p(np.exp(np.minimum(v, 20)))) if softplus else v


def _brute_force(p, M, softplus):
    """out from unrolled sums: forward weight prod_{r=s+1..t} abar_r for s<=t,
    local backward weight prod_{r=t..s-1} abar_r for t<s<=end of t's window."""
    x, A, Bm, Cm = p["x"], p["A"], p["Bm"], p["Cm"]
    Bsz, D, L = x.shape
    N = A.shape[1]
    dt = _timestep(p, softplus)
    out = np.zeros((Bsz, D, L))
    for b in range(Bsz):
        for d in range(D):
            for t in range(L):
                acc = 0.0
                w_end = min(L - 1, (t // M + 1) * M - 1)
                for n in range(N):
                    abar = [math.exp(dt[b, d, r] * A[d, n]) for r in range(L)]
                    u = [dt[b, d, r] * Bm[b, n, r] * x[b, d, r] for r in range(L)]
                    h = 0.0
                    for s in range(0, t + 1):
                        w = 1.0
                        for r in range(s + 1, t + 1):
                            w *= abar[r]
                        h += w * u[s]
                    for s in range(t + 1, w_end + 1):
                        w = 1.0
                        for r in range(t, s):
                            w *= abar[r]
                        h += w * u[s]
                    acc += Cm[b, n, t] * h
                if p["Dskip"] is not None:
                    acc += p["Dskip"][d] * x[b, d, t]
                if p["z"] is not None:
                    zz = p["z"][b, d, t]
                    acc *= zz / (1.0 + math.exp(-zz))
                out[b, d, t] = acc
    return out


@pytest.mark.parametrize("L,M", [(13, 4), (9, 3), (8, 1), (7, 10), (16, 4), (5, 5), (12, 2),
                                 (11, 5), (6, 9), (1, 4), (17, 8)])
def test_forward_matches_unrolled_sums(oracle, L, M):
    p = _rand_problem(2, 3, 3, L, seed=100 + L * 31 + M)
    got = oracle.fwd(**p, window=M, delta_softplus=True)
    ref = _brute_force(p, M, True)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_forward_unrolled_sums_no_softplus_no_optionals(oracle):
    p = _rand_problem(1, 2, 4, 10, softplus=False, gate=False, skip=False, bias=False, seed=5)
    got = oracle.fwd(**p, window=3, delta_softplus=False)
    ref = _brute_force(p, 3, False)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_window_one_is_plain_scan_and_iir_filter(oracle):
    """M = 1: every step closes its own window, the backward part vanishes, and
    Eq. 1-2 with constant delta, A and Bm = Cm = 1 is the one-pole IIR filter
    y_t = r y_{t-1} + delta x_t, r = exp(delta A)."""
    L, dlt, a = 64, 0.07, -1.3
    x = RNG.standard_normal((1, 1, L))
    p = dict(x=x, delta=np.full((1, 1, L), dlt), A=np.array([[a]]),
             Bm=np.ones((1, 1, L)), Cm=np.ones((1, 1, L)))
    got = oracle.fwd(**p, window=1, delta_softplus=False)[0, 0]
    r = math.exp(dlt * a)
    ref = scipy.signal.lfilter([dlt], [1.0, -r], x[0, 0])
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-14)


def test_zero_timestep_gives_skip_times_gate(oracle):
    """delta = 0 => abar = 1, u = 0 => out = Dskip * x * SiLU(z) exactly."""
    p = _rand_problem(2, 4, 5, 19, softplus=False, bias=False, seed=11)
    p["delta"] = np.zeros_like(p["delta"])
    got = oracle.fwd(**p, window=4, delta_softplus=False)
    z = p["z"]
    ref = p["Dskip"][None, :, None] * p["x"] * (z / (1 + np.exp(-z)))
    np.testing.assert_allclose(got, ref, rtol=1e-15, atol=0)


@pytest.mark.parametrize("M", [23, 24, 100])
def test_single_window_relates_to_global_bidirectional(oracle, M):
    """With one window covering the row the local backward state is the global
    backward state of Eq. 4 minus its own input term, so
    lb(M>=L) = bidir(set b := set f) - sum_n Cm u_t - Dskip x_t (ungated)."""
    L = 23
    p = _rand_problem(2, 3, 4, L, gate=False, seed=21)
    lb = oracle.fwd(**p, window=M, delta_softplus=True)
    s = dict(p, delta_softplus=True)
    bi = oracle.bidir_fwd(s, s)
    dt = _timestep(p, True)
    cu = np.einsum("bnl,bdl,bnl,bdl->bdl", p["Cm"], dt, p["Bm"], p["x"])
    ref = bi - cu - p["Dskip"][None, :, None] * p["x"]
    np.testing.assert_allclose(lb, ref, rtol=1e-12, atol=1e-13)


def test_bidirectional_matches_two_unrolled_scans(oracle):
    """Eq. 4-6 from unrolled sums with two independent parameter sets."""
    L = 9
    pf = _rand_problem(1, 2, 3, L, seed=31)
    pb = _rand_problem(1, 2, 3, L, seed=32)
    got = oracle.bidir_fwd(dict(pf, delta_softplus=True), dict(pb, delta_softplus=True))
    ref = np.zeros((1, 2, L))
    for which, p in (("f", pf), ("b", pb)):
        dt = _timestep(p, True)
        for d in range(2):
            for t in range(L):
                acc = p["Dskip"][d] * p["x"][0, d, t]
                for n in range(3):
                    src = range(0, t + 1) if which == "f" else range(t, L)
                    for s in src:
                        lo, hi = (s + 1, t + 1) if which == "f" else (t, s)
                        w = math.exp(sum(dt[0, d, r] for r in range(lo, hi)) * p["A"][d, n])
                        acc += p["Cm"][0, n, t] * w * dt[0, d, s] * p["Bm"][0, n, s] * p["x"][0, d, s]
                ref[0, d, t] += acc
    z = pf["z"]
    ref *= z / (1 + np.exp(-z))
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_bidirectional_is_plain_scan_plus_flipped_plain_scan(oracle):
    L = 37
    pf = _rand_problem(2, 3, 4, L, gate=False, seed=41)
    pb = _rand_problem(2, 3, 4, L, gate=False, seed=42)
    bi = oracle.bidir_fwd(dict(pf, delta_softplus=True), dict(pb, delta_softplus=True))
    fwd = oracle.fwd(**pf, window=1, delta_softplus=True)
    flipped = {k: (v[..., ::-1] if isinstance(v, np.ndarray) and v.ndim == 3 else v)
               for k, v in pb.items()}
    back = oracle.fwd(**flipped, window=1, delta_softplus=True)[..., ::-1]
    np.testing.assert_allclose(bi, fwd + back, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("L,M,s", [(14, 4, 6), (14, 4, 7), (14, 4, 4), (14, 4, 13), (10, 5, 9), (9, 3, 0)])
def test_impulse_response_and_window_locality(oracle, L, M, s):
    """x = unit impulse at s: to the right the response is the plain forward
    kernel; to the left it is non-zero only inside s's window, with the decay
    product over steps t..s-1 (destination's own abar included)."""
    r = np.random.default_rng(50 + s)
    N = 3
    dt = r.uniform(0.05, 0.4, size=L)
    A = -r.uniform(0.5, 2.0, size=(1, N))
    Bm = r.standard_normal((1, N, L))
    Cm = r.standard_normal((1, N, L))
    x = np.zeros((1, 1, L))
    x[0, 0, s] = 1.0
    got = oracle.fwd(x=x, delta=dt[None, None, :], A=A, Bm=Bm, Cm=Cm, window=M,
                     delta_softplus=False)[0, 0]
    S = np.concatenate([[0.0], np.cumsum(dt)])       # S[k] = sum of dt[0..k-1]
    for t in range(L):
        if t >= s:
            ref = sum(Cm[0, n, t] * math.exp(A[0, n] * (S[t + 1] - S[s + 1])) * dt[s] * Bm[0, n, s]
                      for n in range(N))
        elif t // M == s // M:
            ref = sum(Cm[0, n, t] * math.exp(A[0, n] * (S[s] - S[t])) * dt[s] * Bm[0, n, s]
                      for n in range(N))
        else:
            ref = 0.0
            assert got[t] == 0.0
        assert got[t] == pytest.approx(ref, rel=1e-12, abs=1e-15)


def test_closed_form_constant_coefficients(oracle):
    """Constant delta, Bm = Cm = x = 1, one window: h_t is two geometric sums and
    is symmetric under t <-> L-1-t."""
    L, dlt, a = 33, 0.11, -0.9
    r = math.exp(dlt * a)
    p = dict(x=np.ones((1, 1, L)), delta=np.full((1, 1, L), dlt), A=np.array([[a]]),
             Bm=np.ones((1, 1, L)), Cm=np.ones((1, 1, L)))
    got = oracle.fwd(**p, window=L, delta_softplus=False)[0, 0]
    t = np.arange(L)
    ref = dlt * ((1 - r ** (t + 1)) + r * (1 - r ** (L - 1 - t))) / (1 - r)
    np.testing.assert_allclose(got, ref, rtol=1e-12)
    np.testing.assert_allclose(got, got[::-1], rtol=1e-12)


def test_local_backward_is_flipped_plain_scan_per_window(oracle):
    """Inside each window, g + u equals flip(plain_scan(flip(abar), flip(u))):
    the local backward scan is the forward scan run right to left."""
    L, M = 22, 4
    p = _rand_problem(1, 2, 3, L, gate=False, skip=False, seed=61)
    lb = oracle.fwd(**p, window=M, delta_softplus=True)
    plain = oracle.fwd(**p, window=1, delta_softplus=True)
    dt = _timestep(p, True)
    cu = np.einsum("bnl,bdl,bnl,bdl->bdl", p["Cm"], dt, p["Bm"], p["x"])
    ref = np.zeros_like(lb)
    for w0 in range(0, L, M):
        w1 = min(L, w0 + M)
        sub = {k: (v[..., w0:w1][..., ::-1] if isinstance(v, np.ndarray) and v.ndim == 3 else v)
               for k, v in p.items()}
        ref[..., w0:w1] = oracle.fwd(**sub, window=1, delta_softplus=True)[..., ::-1]
    np.testing.assert_allclose(lb - plain, ref - cu, rtol=1e-11, atol=1e-13)


def test_output_is_linear_in_x(oracle):
    p = _rand_problem(1, 3, 4, 21, gate=False, seed=71)
    x1, x2 = p["x"], np.random.default_rng(72).standard_normal(p["x"].shape)
    f = lambda xx: oracle.fwd(**dict(p, x=xx), window=4, delta_softplus=True)
    np.testing.assert_allclose(f(2.5 * x1 - 0.75 * x2), 2.5 * f(x1) - 0.75 * f(x2),
                               rtol=1e-11, atol=1e-12)


def test_ragged_tail_equals_zero_padding(oracle):
    """A short last window behaves like padding with delta = 0 steps."""
    L, M, pad = 13, 4, 3
    p = _rand_problem(1, 2, 3, L, softplus=False, bias=False, seed=81)
    base = oracle.fwd(**p, window=M, delta_softplus=False)
    q = dict(p)
    for k in ("x", "delta", "Bm", "Cm", "z"):
        fill = np.zeros(p[k].shape[:-1] + (pad,))
        if k in ("Bm", "Cm", "z", "x"):
            fill = np.random.default_rng(82).standard_normal(fill.shape)
        if k == "delta":
            fill = np.zeros_like(fill)
        q[k] = np.concatenate([p[k], fill], axis=-1)
    padded = oracle.fwd(**q, window=M, delta_softplus=False)
    np.testing.assert_allclose(padded[..., :L], base, rtol=1e-13, atol=1e-15)


# ------------------------------------------- the time step above and below 20

def _const_step_problem(v, L=9, seed=0):
    """Every time step has delta + delta_bias = v exactly; A is small so that
    abar stays away from zero at time steps near 20."""
    r = np.random.default_rng(300 + seed)
    B, D, N = 1, 2, 3
    bias = np.array([0.5, -1.25])
    return dict(
        x=r.standard_normal((B, D, L)),
        delta=np.broadcast_to((v - bias)[None, :, None], (B, D, L)).copy(),
        A=-r.uniform(0.005, 0.02, size=(D, N)),
        Bm=r.standard_normal((B, N, L)), Cm=r.standard_normal((B, N, L)),
        Dskip=r.standard_normal(D), z=r.standard_normal((B, D, L)), delta_bias=bias)


@pytest.mark.parametrize("v", [20.5, 25.0, 40.0])
def test_softplus_is_identity_above_twenty(oracle, v):
    """Algorithm 1's Delta line with the reading softplus(v) = v for v > 20: the
    run with softplus on equals the run with softplus off bit for bit (and so do
    the gradients, whose softplus factor is exactly 1 there)."""
    p = _const_step_problem(v, seed=int(v))
    assert np.all(p["delta"] + p["delta_bias"][None, :, None] == v)
    on = oracle.fwd(**p, window=4, delta_softplus=True)
    off = oracle.fwd(**p, window=4, delta_softplus=False)
    assert np.array_equal(on, off)
    dout = np.random.default_rng(5).standard_normal(p["x"].shape)
    g_on = oracle.bwd(**p, dout=dout, window=4, delta_softplus=True)
    g_off = oracle.bwd(**p, dout=dout, window=4, delta_softplus=False)
    for k in g_on:
        assert np.array_equal(g_on[k], g_off[k]), k


@pytest.mark.parametrize("v", [19.0, 19.99, 20.0])
def test_softplus_is_log1p_exp_up_to_twenty(oracle, v):
    """At and below 20 the time step is log(1 + exp(v)) itself (no threshold in
    this check): the output equals the unrolled sums fed with it, differs from
    the softplus-off run, and ddelta carries the factor sigma(v) < 1."""
    p = _const_step_problem(v, seed=int(v * 100))
    sp = math.log1p(math.exp(v))
    assert sp > v
    on = oracle.fwd(**p, window=4, delta_softplus=True)
    q = dict(p, delta=np.full_like(p["delta"], sp), delta_bias=None)
    ref = _brute_force(q, 4, False)
    np.testing.assert_allclose(on, ref, rtol=1e-13, atol=1e-14)
    assert not np.array_equal(on, oracle.fwd(**p, window=4, delta_softplus=False))
    dout = np.random.default_rng(6).standard_normal(p["x"].shape)
    g_on = oracle.bwd(**p, dout=dout, window=4, delta_softplus=True)
    g_lin = oracle.bwd(**q, dout=dout, window=4, delta_softplus=False)
    sig = 1.0 / (1.0 + math.exp(-v))
    assert sig < 1.0
    np.testing.assert_allclose(g_on["ddelta"], g_lin["ddelta"] * sig, rtol=1e-13, atol=1e-300)
    np.testing.assert_allclose(g_on["ddelta_bias"], g_lin["ddelta"].sum(axis=(0, 2)) * sig, rtol=1e-12)
    # sigma(19) = 1 - 5.6e-9 is told apart from 1 at this tolerance
    assert np.max(np.abs(g_on["ddelta"] - g_lin["ddelta"])) > 1e-10 * np.max(np.abs(g_lin["ddelta"]))


@pytest.mark.parametrize("v", [18.0, 19.5, 20.5, 22.0])
def test_time_step_gradients_by_central_differences_around_twenty(oracle, v):
    p = _const_step_problem(v, L=7, seed=int(v * 10))
    dout = np.random.default_rng(7).standard_normal(p["x"].shape)
    g = oracle.bwd(**p, dout=dout, window=4, delta_softplus=True)
    loss = lambda q: float(np.sum(dout * oracle.fwd(**q, window=4, delta_softplus=True)))
    h = 1e-5
    for name, gname in (("delta", "ddelta"), ("delta_bias", "ddelta_bias")):
        arr = p[name]
        scale = np.sqrt(np.mean(g[gname] ** 2))
        for fi in range(0, arr.size, max(1, arr.size // 6)):
            idx = np.unravel_index(fi, arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += h
            lo[idx] -= h
            fd = (loss(dict(p, **{name: hi})) - loss(dict(p, **{name: lo}))) / (2 * h)
            assert abs(fd - g[gname][idx]) <= 1e-6 * max(abs(fd), scale), (name, idx, fd, g[gname][idx])


# ----------------------------------------------------------------- gradients

_GRAD_OF = dict(x="dx", delta="ddelta", z="dz", Bm="dBm", Cm="dCm", A="dA", Dskip="dDskip",
                delta_bias="ddelta_bias")


@pytest.mark.parametrize("L,M,softplus", [(13, 4, True), (9, 3, True), (8, 1, True), (7, 10, False),
                                          (16, 4, False), (5, 5, True)])
def test_gradients_match_central_differences(oracle, L, M, softplus):
    p = _rand_problem(2, 3, 3, L, softplus=softplus, seed=900 + L)
    dout = np.random.default_rng(901 + L).standard_normal(p["x"].shape)
    g = oracle.bwd(**p, dout=dout, window=M, delta_softplus=softplus)
    loss = lambda q: float(np.sum(dout * oracle.fwd(**q, window=M, delta_softplus=softplus)))
    h = 1e-6
    r = np.random.default_rng(902 + L)
    for name, gname in _GRAD_OF.items():
        arr = p[name]
        flat_idx = r.choice(arr.size, size=min(arr.size, 12), replace=False)
        scale = np.sqrt(np.mean(g[gname] ** 2)) + 1e-30
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += h
            lo[idx] -= h
            fd = (loss(dict(p, **{name: hi})) - loss(dict(p, **{name: lo}))) / (2 * h)
            assert abs(fd - g[gname][idx]) <= 2e-6 * max(abs(fd), scale), (name, idx, fd, g[gname][idx])


def test_gradients_without_optionals(oracle):
    p = _rand_problem(1, 2, 2, 11, gate=False, skip=False, bias=False, seed=950)
    dout = np.random.default_rng(951).standard_normal(p["x"].shape)
    g = oracle.bwd(**p, dout=dout, window=4, delta_softplus=True)
    assert g["dz"] is None
    loss = lambda q: float(np.sum(dout * oracle.fwd(**q, window=4, delta_softplus=True)))
    h = 1e-6
    for name in ("x", "delta", "Bm", "Cm", "A"):
        arr = p[name]
        for fi in range(0, arr.size, max(1, arr.size // 7)):
            idx = np.unravel_index(fi, arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += h
            lo[idx] -= h
            fd = (loss(dict(p, **{name: hi})) - loss(dict(p, **{name: lo}))) / (2 * h)
            assert fd == pytest.approx(g[_GRAD_OF[name]][idx], rel=2e-6, abs=1e-8)


def test_adjoint_identity_in_x(oracle):
    """out is linear in x (no gate): <dout, J v> = <J^T dout, v>."""
    p = _rand_problem(2, 3, 4, 19, gate=False, seed=960)
    r = np.random.default_rng(961)
    v, dout = r.standard_normal(p["x"].shape), r.standard_normal(p["x"].shape)
    Jv = oracle.fwd(**dict(p, x=v), window=4, delta_softplus=True)
    g = oracle.bwd(**p, dout=dout, window=4, delta_softplus=True)
    assert float(np.sum(dout * Jv)) == pytest.approx(float(np.sum(g["dx"] * v)), rel=1e-11)


def test_oracle_rejects_bad_window(oracle):
    p = _rand_problem(1, 1, 1, 4, seed=1)
    with pytest.raises(RuntimeError):
        oracle.fwd(**p, window=0, delta_softplus=True)


def test_empty_inputs(oracle):
    p = _rand_problem(1, 2, 3, 0, seed=2)
    assert oracle.fwd(**p, window=4, delta_softplus=True).shape == (1, 2, 0)


def test_oracle_reproduces_its_frozen_small_case(oracle):
    """Regression fixture written by tests/golden/make_golden.py from the oracle
    (not a value from the paper, which prints none)."""
    import importlib.util
    import json
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    gold = json.load(open(os.path.join(here, "golden", "lbscan_small_golden.json")))
    p = mg.small_problem()
    np.testing.assert_allclose(oracle.fwd(**p, window=gold["window"]), np.array(gold["fwd"]), rtol=1e-13)
    np.testing.assert_allclose(oracle.bidir_fwd(dict(p), dict(p)), np.array(gold["bidir_self"]), rtol=1e-13)
    dout = np.random.default_rng(424243).standard_normal(p["x"].shape)
    g = oracle.bwd(**p, dout=dout, window=gold["window"])
    for k, v in gold["bwd"].items():
        np.testing.assert_allclose(g[k], np.array(v), rtol=1e-12, atol=1e-14)
