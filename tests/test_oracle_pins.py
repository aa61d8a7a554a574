"""Pins of the CPU oracle to things other than itself (CPU only).

Each test fixes one part of the oracle to a closed form, a library routine, a special
case the paper states, or brute force, so that a dropped term, a wrong sign or index,
or a transposed operand fails at least one of them.
"""
import os

import numpy as np
import pytest
from scipy.special import expit

from oracle import ss_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, B=2, D=3, L=9, N=4):
    rng = np.random.default_rng(seed)
    return dict(
        u=rng.normal(size=(B, D, L)), delta=rng.normal(size=(B, D, L)),
        z=rng.normal(size=(B, D, L)), A=-np.abs(rng.normal(size=(D, N))) - 0.1,
        Bm=rng.normal(size=(B, N, L)), Cm=rng.normal(size=(B, N, L)),
        Dskip=rng.normal(size=D), bias=rng.normal(size=D), h0=rng.normal(size=(B, D, N)))


# ---------------------------------------------------------------- Eq. 3: LTI closed form
@pytest.mark.parametrize("exact_zoh", [False, True])
def test_lti_equals_convolution_kernel(exact_zoh):
    """Constant (delta, B, C): y = x * K with K_k = C Abar^k Bbar (Eq. 3a/3b)."""
    rng = np.random.default_rng(1)
    B, D, L, N = 2, 3, 40, 5
    u = rng.normal(size=(B, D, L))
    dt = rng.uniform(0.05, 0.8, size=D)
    A = -rng.uniform(0.2, 3.0, size=(D, N))
    Bn = rng.normal(size=(B, N))
    Cn = rng.normal(size=(B, N))
    Dskip = rng.normal(size=D)
    delta = np.broadcast_to(dt[None, :, None], (B, D, L))
    Bm = np.broadcast_to(Bn[:, :, None], (B, N, L))
    Cm = np.broadcast_to(Cn[:, :, None], (B, N, L))
    got = orc.scan_fwd(u, delta, A, Bm, Cm, Dskip=Dskip, exact_zoh=exact_zoh)["out"]
    want = np.zeros_like(u)
    for b in range(B):
        for d in range(D):
            abar = np.exp(dt[d] * A[d])
            bbar = (abar - 1.0) / A[d] * Bn[b] if exact_zoh else dt[d] * Bn[b]
            K = np.array([np.sum(Cn[b] * abar ** k * bbar) for k in range(L)])
            want[b, d] = np.convolve(u[b, d], K)[:L] + Dskip[d] * u[b, d]
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)


# ------------------------------------------------- Eq. 2a unrolled: brute-force products
def test_time_varying_states_bruteforce():
    """h_t = sum_{s<=t} (prod_{r=s+1..t} abar_r) bbar_s u_s + (prod_{r<=t} abar_r) h0."""
    p = _rand(2, B=2, D=2, L=11, N=3)
    delta = np.abs(p["delta"]) * 0.3
    got = orc.scan_fwd(p["u"], delta, p["A"], p["Bm"], p["Cm"], h0=p["h0"])
    B, D, L = p["u"].shape
    N = p["A"].shape[1]
    y = np.zeros((B, D, L))
    hl = np.zeros((B, D, N))
    for b in range(B):
        for d in range(D):
            abar = np.exp(delta[b, d][:, None] * p["A"][d][None, :])      # (L,N)
            bu = delta[b, d][:, None] * p["Bm"][b].T * p["u"][b, d][:, None]  # (L,N)
            for t in range(L):
                h = np.prod(abar[: t + 1], axis=0) * p["h0"][b, d]
                for s in range(t + 1):
                    h = h + np.prod(abar[s + 1: t + 1], axis=0) * bu[s]
                y[b, d, t] = np.dot(p["Cm"][b, :, t], h)
            hl[b, d] = h
    np.testing.assert_allclose(got["out"], y, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(got["h_last"], hl, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------- A = 0: textbook prefix sum
def test_A_zero_is_cumulative_sum():
    p = _rand(3)
    A0 = np.zeros_like(p["A"])
    delta = np.abs(p["delta"])
    got = orc.scan_fwd(p["u"], delta, A0, p["Bm"], p["Cm"])
    # h[b,d,n,t] = cumsum_t(delta*u * B)
    h = np.cumsum((delta * p["u"])[:, :, None, :] * p["Bm"][:, None, :, :], axis=-1)
    y = np.einsum("bnt,bdnt->bdt", p["Cm"], h)
    np.testing.assert_allclose(got["out"], y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got["h_last"], h[..., -1], rtol=1e-12, atol=1e-13)
    # exact ZOH has the same A -> 0 limit
    got2 = orc.scan_fwd(p["u"], delta, A0, p["Bm"], p["Cm"], exact_zoh=True)
    np.testing.assert_allclose(got2["out"], y, rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------- Theorem 1
def test_theorem1_gate_decay_factor():
    """N=1, A=-1, softplus: Abar_t = 1 - sigmoid(r_t) in both B-bar modes (proof of Thm 1)."""
    rng = np.random.default_rng(4)
    L = 12
    r = rng.normal(size=(1, 1, L)) * 2.0
    bias = np.array([0.3])
    zero_u = np.zeros((1, 1, L))
    A = -np.ones((1, 1))
    ones = np.ones((1, 1, L))
    for exact in (False, True):
        got = orc.scan_fwd(zero_u, r, A, ones, ones, bias=bias, h0=np.ones((1, 1, 1)),
                           softplus=True, exact_zoh=exact)["out"][0, 0]
        want = np.cumprod(1.0 - expit(r[0, 0] + bias[0]))
        np.testing.assert_allclose(got, want, rtol=1e-12)


def test_theorem1_full_gated_recurrence():
    """Exact ZOH, B=C=1: h_t = (1-g_t) h_{t-1} + g_t x_t, g_t = sigmoid(r_t) (Eq. 5)."""
    rng = np.random.default_rng(5)
    L = 30
    r = rng.normal(size=L) * 1.5
    x = rng.normal(size=L)
    g = expit(r)
    h, want = 0.0, []
    for t in range(L):
        h = (1 - g[t]) * h + g[t] * x[t]
        want.append(h)
    ones = np.ones((1, 1, L))
    got = orc.scan_fwd(x[None, None], r[None, None], -np.ones((1, 1)), ones, ones,
                       softplus=True, exact_zoh=True)["out"][0, 0]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    # first-order B-bar differs from it exactly by the input weight softplus(r) vs sigmoid(r)
    got1 = orc.scan_fwd(x[None, None], r[None, None], -np.ones((1, 1)), ones, ones,
                        softplus=True)["out"][0, 0]
    h, want1 = 0.0, []
    for t in range(L):
        h = (1 - g[t]) * h + np.logaddexp(0.0, r[t]) * x[t]
        want1.append(h)
    np.testing.assert_allclose(got1, want1, rtol=1e-12, atol=1e-14)


def test_theorem1_hand_worked_fixture():
    rows = np.loadtxt(os.path.join(GOLDEN, "theorem1_gate.txt"))
    x, want = rows[:, 1], rows[:, 2]
    L = len(x)
    ones = np.ones((1, 1, L))
    got = orc.scan_fwd(x[None, None], np.zeros((1, 1, L)), -np.ones((1, 1)), ones, ones,
                       softplus=True, exact_zoh=True)["out"][0, 0]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-15)


def test_softplus_matches_library_logaddexp():
    r = np.array([-800.0, -30.0, -1.0, 0.0, 1.0, 30.0, 800.0])
    L = len(r)
    # N=1, A=0, B=C=1, u=1, h0=0  ->  out_t = cumsum(softplus(r))
    ones = np.ones((1, 1, L))
    got = orc.scan_fwd(ones, r[None, None], np.zeros((1, 1)), ones, ones, softplus=True)["out"][0, 0]
    np.testing.assert_allclose(np.diff(np.concatenate([[0.0], got])), np.logaddexp(0.0, r),
                               rtol=1e-12, atol=1e-300)


# ------------------------------------------------- Section 3.5.2: large / small step size
def test_large_step_resets_and_zero_step_persists():
    p = _rand(6, B=1, D=2, L=6, N=3)
    p["A"] = p["A"] - 1.0          # every |A| >= 1, so exp(60*A) is below 1e-26
    big = np.full_like(p["delta"], 60.0)
    # exact ZOH: Abar -> 0 and Bbar -> -B/A, so the state forgets everything but x_t
    got = orc.scan_fwd(p["u"], big, p["A"], p["Bm"], p["Cm"], h0=p["h0"], exact_zoh=True)
    want_h = -p["Bm"][0, :, -1][None, :] / p["A"] * p["u"][0, :, -1][:, None]
    np.testing.assert_allclose(got["h_last"][0], want_h, rtol=1e-9)
    # first-order rule: h_t -> delta * B_t * u_t
    got = orc.scan_fwd(p["u"], big, p["A"], p["Bm"], p["Cm"], h0=p["h0"])
    want_h = 60.0 * p["Bm"][0, :, -1][None, :] * p["u"][0, :, -1][:, None]
    np.testing.assert_allclose(got["h_last"][0], want_h, rtol=1e-9)
    # delta = 0: the state persists and the input is ignored
    zero = np.zeros_like(p["delta"])
    got = orc.scan_fwd(p["u"], zero, p["A"], p["Bm"], p["Cm"], h0=p["h0"], Dskip=p["Dskip"])
    np.testing.assert_allclose(got["h_last"], p["h0"][:1], rtol=0, atol=0)
    want = np.einsum("nt,dn->dt", p["Cm"][0], p["h0"][0]) + p["Dskip"][:, None] * p["u"][0]
    np.testing.assert_allclose(got["out"][0], want, rtol=1e-12, atol=1e-13)


# -------------------------------------- Appendix D chunking; Section 2 recurrent == scan
def _full(p, **kw):
    return orc.scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dskip=p["Dskip"],
                        z=p["z"], bias=p["bias"], softplus=True, **kw)


def test_chunk_continuation_and_last_state():
    p = _rand(7, L=23)
    whole = _full(p, h0=p["h0"])
    for cut in (1, 8, 22):
        a = orc.scan_fwd(p["u"][..., :cut], p["delta"][..., :cut], p["A"], p["Bm"][..., :cut],
                         p["Cm"][..., :cut], Dskip=p["Dskip"], z=p["z"][..., :cut],
                         bias=p["bias"], h0=p["h0"], softplus=True)
        b = orc.scan_fwd(p["u"][..., cut:], p["delta"][..., cut:], p["A"], p["Bm"][..., cut:],
                         p["Cm"][..., cut:], Dskip=p["Dskip"], z=p["z"][..., cut:],
                         bias=p["bias"], h0=a["h_last"], softplus=True)
        np.testing.assert_allclose(np.concatenate([a["out"], b["out"]], -1), whole["out"],
                                   rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(b["h_last"], whole["h_last"], rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("exact_zoh", [False, True])
def test_step_by_step_equals_scan(exact_zoh):
    p = _rand(8, L=10)
    whole = _full(p, h0=p["h0"], exact_zoh=exact_zoh)
    h = p["h0"].copy()
    for t in range(p["u"].shape[-1]):
        out_t, h = orc.step(h, p["u"][..., t], p["delta"][..., t], p["A"], p["Bm"][..., t],
                            p["Cm"][..., t], Dskip=p["Dskip"], z_t=p["z"][..., t],
                            bias=p["bias"], softplus=True, exact_zoh=exact_zoh)
        np.testing.assert_allclose(out_t, whole["out"][..., t], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(h, whole["h_last"], rtol=1e-13, atol=1e-14)


# ------------------------------------------------------------------ structural properties
def test_causality():
    p = _rand(9, L=12)
    base = _full(p)["out"]
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    for k in ("u", "delta", "z", "Bm", "Cm"):
        q[k][..., 7:] += 1.0
    pert = _full(q)["out"]
    np.testing.assert_array_equal(base[..., :7], pert[..., :7])
    assert np.all(base[..., 7:] != pert[..., 7:])


def test_linearity_in_u_and_h0_without_gate():
    p = _rand(10)
    kw = dict(Dskip=p["Dskip"], bias=p["bias"], softplus=True)
    f = lambda u, h0: orc.scan_fwd(u, p["delta"], p["A"], p["Bm"], p["Cm"], h0=h0, **kw)["out"]
    u2 = np.random.default_rng(11).normal(size=p["u"].shape)
    lhs = f(2.0 * p["u"] - 3.0 * u2, 2.0 * p["h0"])
    rhs = 2.0 * f(p["u"], p["h0"]) - 3.0 * f(u2, np.zeros_like(p["h0"]))
    np.testing.assert_allclose(lhs, rhs, rtol=1e-11, atol=1e-12)


def test_channel_and_batch_independence():
    p = _rand(12, B=3, D=4)
    base = _full(p, h0=p["h0"])
    pd = np.array([2, 0, 3, 1])
    pb = np.array([1, 2, 0])
    q = dict(u=p["u"][pb][:, pd], delta=p["delta"][pb][:, pd], z=p["z"][pb][:, pd],
             A=p["A"][pd], Bm=p["Bm"][pb], Cm=p["Cm"][pb], Dskip=p["Dskip"][pd],
             bias=p["bias"][pd], h0=p["h0"][pb][:, pd])
    perm = _full(q, h0=q["h0"])
    np.testing.assert_array_equal(perm["out"], base["out"][pb][:, pd])
    np.testing.assert_array_equal(perm["h_last"], base["h_last"][pb][:, pd])
    # state index n is a dummy: permuting it in A, B, C, h0 changes y only by rounding order
    pn = np.array([3, 1, 0, 2])
    r = orc.scan_fwd(p["u"], p["delta"], p["A"][:, pn], p["Bm"][:, pn], p["Cm"][:, pn],
                     Dskip=p["Dskip"], z=p["z"], bias=p["bias"], h0=p["h0"][..., pn], softplus=True)
    np.testing.assert_allclose(r["out"], base["out"], rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(r["h_last"], base["h_last"][..., pn])


def test_gate_skip_and_bias_enter_as_stated():
    p = _rand(13)
    kw = dict(bias=p["bias"], softplus=True)
    plain = orc.scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], **kw)
    np.testing.assert_array_equal(plain["out"], plain["y_pre"])
    skip = orc.scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dskip=p["Dskip"], **kw)
    np.testing.assert_allclose(skip["out"] - plain["out"], p["Dskip"][None, :, None] * p["u"],
                               rtol=1e-10, atol=1e-12)
    gated = orc.scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dskip=p["Dskip"],
                         z=p["z"], **kw)
    np.testing.assert_allclose(gated["out"], skip["out"] * p["z"] * expit(p["z"]), rtol=1e-12)
    np.testing.assert_array_equal(gated["y_pre"], skip["out"])
    # bias is added to the raw step input before softplus
    folded = orc.scan_fwd(p["u"], p["delta"] + p["bias"][None, :, None], p["A"], p["Bm"],
                          p["Cm"], softplus=True)
    np.testing.assert_allclose(folded["out"], plain["out"], rtol=1e-12, atol=1e-14)
    # softplus off: delta is used as given
    raw = orc.scan_fwd(p["u"], np.logaddexp(0.0, p["delta"] + p["bias"][None, :, None]),
                       p["A"], p["Bm"], p["Cm"])
    np.testing.assert_allclose(raw["out"], plain["out"], rtol=1e-12, atol=1e-14)


# ------------------------------------------- independent vectorised numpy re-implementation
def _numpy_scan(p, exact_zoh=False):
    dt = np.logaddexp(0.0, p["delta"] + p["bias"][None, :, None])
    h = p["h0"].copy()
    outs = []
    for t in range(p["u"].shape[-1]):
        da = dt[..., t, None] * p["A"][None]
        abar = np.exp(da)
        phi = np.where(p["A"][None] != 0, np.expm1(da) / p["A"][None], dt[..., t, None]) if exact_zoh \
            else dt[..., t, None]
        h = abar * h + phi * p["Bm"][:, None, :, t] * p["u"][..., t, None]
        y = np.sum(h * p["Cm"][:, None, :, t], -1) + p["Dskip"][None] * p["u"][..., t]
        outs.append(y * p["z"][..., t] * expit(p["z"][..., t]))
    return np.stack(outs, -1), h


@pytest.mark.parametrize("exact_zoh", [False, True])
def test_against_independent_numpy_loop(exact_zoh):
    p = _rand(14, B=2, D=5, L=65, N=16)
    got = _full(p, h0=p["h0"], exact_zoh=exact_zoh)
    out, h = _numpy_scan(p, exact_zoh)
    np.testing.assert_allclose(got["out"], out, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(got["h_last"], h, rtol=1e-11, atol=1e-12)


def test_threads_do_not_change_result():
    p = _rand(15, B=3, D=7, L=33, N=4)
    a = _full(p, nthreads=1)
    b = _full(p, nthreads=4)
    np.testing.assert_array_equal(a["out"], b["out"])


def test_oracle_matches_its_stored_fixture():
    """Regression guard: the oracle still produces the numbers stored by
    tests/golden/make_oracle_fixture.py (its own earlier output, not an independent pin)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_oracle_fixture", os.path.join(GOLDEN, "make_oracle_fixture.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    w = mod.case()
    now = {False: mod.compute(w, False), True: mod.compute(w, True)}
    seen = 0
    for line in open(os.path.join(GOLDEN, "oracle_tiny_case.txt")):
        if line.startswith("#"):
            continue
        name, mode, *vals = line.split()
        got = np.asarray(now[mode == "zoh"][name]).reshape(-1)
        np.testing.assert_allclose(got, np.array(vals, dtype=np.float64), rtol=1e-13, atol=1e-15, err_msg=name + " " + mode)
        seen += 1
    assert seen == 20
