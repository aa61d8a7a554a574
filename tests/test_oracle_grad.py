"""Pins of the oracle's backward pass (CPU only).

The paper gives no gradient formulas (Appendix D only says states are recomputed), so
the oracle's reverse sweep is pinned to the forward oracle itself, which the other test
file pins to closed forms: central finite differences on single coordinates of every
input, directional derivatives over whole tensors, and special cases whose gradient is
known in closed form.
"""
import numpy as np
import pytest

from oracle import ss_oracle as orc

NAMES = ["u", "delta", "z", "Bm", "Cm", "A", "Dskip", "bias", "h0"]
GRAD_OF = {"u": "du", "delta": "ddelta", "z": "dz", "Bm": "dB", "Cm": "dC", "A": "dA",
           "Dskip": "dD", "bias": "dbias", "h0": "dh0"}


def _problem(seed, B=2, D=3, L=7, N=4):
    rng = np.random.default_rng(seed)
    p = dict(
        u=rng.normal(size=(B, D, L)), delta=rng.normal(size=(B, D, L)) * 0.7,
        z=rng.normal(size=(B, D, L)), A=-np.abs(rng.normal(size=(D, N))) - 0.2,
        Bm=rng.normal(size=(B, N, L)), Cm=rng.normal(size=(B, N, L)),
        Dskip=rng.normal(size=D), bias=rng.normal(size=D) * 0.5,
        h0=rng.normal(size=(B, D, N)))
    W = rng.normal(size=(B, D, L))
    V = rng.normal(size=(B, D, N))
    return p, W, V


def _loss(p, W, V, softplus, exact_zoh, use=("z", "Dskip", "bias", "h0")):
    r = orc.scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"],
                     Dskip=p["Dskip"] if "Dskip" in use else None,
                     z=p["z"] if "z" in use else None,
                     bias=p["bias"] if "bias" in use else None,
                     h0=p["h0"] if "h0" in use else None,
                     softplus=softplus, exact_zoh=exact_zoh, nthreads=1)
    return float(np.sum(r["out"] * W) + np.sum(r["h_last"] * V))


def _grads(p, W, V, softplus, exact_zoh, use=("z", "Dskip", "bias", "h0")):
    return orc.scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], W,
                        Dskip=p["Dskip"] if "Dskip" in use else None,
                        z=p["z"] if "z" in use else None,
                        bias=p["bias"] if "bias" in use else None,
                        h0=p["h0"] if "h0" in use else None,
                        dh_last=V, softplus=softplus, exact_zoh=exact_zoh)


@pytest.mark.parametrize("softplus", [True, False])
@pytest.mark.parametrize("exact_zoh", [False, True])
def test_every_gradient_by_central_differences(softplus, exact_zoh):
    p, W, V = _problem(20)
    if not softplus:
        p["delta"] = np.abs(p["delta"]) + 0.05
        p["bias"] = np.abs(p["bias"])
    g = _grads(p, W, V, softplus, exact_zoh)
    rng = np.random.default_rng(21)
    eps = 1e-6
    for name in NAMES:
        ga = g[GRAD_OF[name]]
        assert ga.shape == p[name].shape
        flat = p[name].reshape(-1)
        idx = rng.choice(flat.size, size=min(flat.size, 12), replace=False)
        for i in idx:
            keep = flat[i]
            flat[i] = keep + eps
            lp = _loss(p, W, V, softplus, exact_zoh)
            flat[i] = keep - eps
            lm = _loss(p, W, V, softplus, exact_zoh)
            flat[i] = keep
            fd = (lp - lm) / (2 * eps)
            an = ga.reshape(-1)[i]
            assert abs(fd - an) <= 2e-7 * max(1.0, abs(fd)), (name, i, fd, an)


@pytest.mark.parametrize("use", [(), ("z",), ("Dskip", "bias"), ("h0",)])
def test_directional_derivative_with_optional_inputs(use):
    """<grad, v> equals the derivative of the loss along a random direction v."""
    p, W, V = _problem(22, B=2, D=4, L=19, N=5)
    g = _grads(p, W, V, True, False, use)
    active = ["u", "delta", "Bm", "Cm", "A"] + list(use)
    rng = np.random.default_rng(23)
    v = {k: rng.normal(size=p[k].shape) for k in active}
    eps = 1e-6
    plus = {k: (p[k] + eps * v[k] if k in v else p[k]) for k in p}
    minus = {k: (p[k] - eps * v[k] if k in v else p[k]) for k in p}
    fd = (_loss(plus, W, V, True, False, use) - _loss(minus, W, V, True, False, use)) / (2 * eps)
    an = sum(float(np.sum(g[GRAD_OF[k]] * v[k])) for k in active)
    assert abs(fd - an) <= 1e-7 * max(1.0, abs(fd))
    for k in ("z", "Dskip", "bias"):
        if k not in use:
            assert g[GRAD_OF[k]] is None


def test_gradient_closed_form_A_zero():
    """A = 0, no gate: y_t = sum_n C_n,t sum_{s<=t} delta_s B_n,s u_s, so
    du_s = delta_s * sum_n B_n,s * sum_{t>=s} C_n,t dout_t (a reversed cumulative sum)."""
    p, W, V = _problem(24, B=1, D=2, L=13, N=3)
    p["A"][:] = 0.0
    delta = np.abs(p["delta"]) + 0.1
    g = orc.scan_bwd(p["u"], delta, p["A"], p["Bm"], p["Cm"], W)
    G = np.flip(np.cumsum(np.flip(p["Cm"][:, None] * W[:, :, None, :], -1), -1), -1)  # (B,D,N,L)
    want_du = delta * np.sum(p["Bm"][:, None] * G, axis=2)
    want_ddelta = p["u"] * np.sum(p["Bm"][:, None] * G, axis=2)
    want_dB = np.sum((delta * p["u"])[:, :, None, :] * G, axis=1)
    H = np.cumsum((delta * p["u"])[:, :, None, :] * p["Bm"][:, None], -1)
    want_dC = np.sum(H * W[:, :, None, :], axis=1)
    np.testing.assert_allclose(g["du"], want_du, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["ddelta"], want_ddelta, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["dB"], want_dB, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["dC"], want_dC, rtol=1e-12, atol=1e-13)


def test_gradient_is_linear_in_dout_and_dh_last():
    p, W, V = _problem(25)
    W2 = np.random.default_rng(26).normal(size=W.shape)
    a = _grads(p, W, V, True, False)
    b = _grads(p, W2, np.zeros_like(V), True, False)
    c = _grads(p, 2 * W - W2, 2 * V, True, False)
    for k in a:
        np.testing.assert_allclose(c[k], 2 * a[k] - b[k], rtol=1e-10, atol=1e-11)


def test_backward_threads_do_not_change_result_beyond_rounding():
    p, W, V = _problem(27, B=3, D=9, L=31, N=4)
    kw = dict(Dskip=p["Dskip"], z=p["z"], bias=p["bias"], h0=p["h0"], dh_last=V, softplus=True)
    a = orc.scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], W, nthreads=1, **kw)
    b = orc.scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], W, nthreads=5, **kw)
    for k in a:
        np.testing.assert_allclose(a[k], b[k], rtol=1e-12, atol=1e-13)
