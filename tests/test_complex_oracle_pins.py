"""Pins of the complex-state oracle (CPU only).

The paper gives the complex case only through its initialisation (Section 3.6: S4D-Lin,
A_n = -1/2 + n i) and the equations of Section 2, so the oracle is pinned to what those fix:
the convolution form of Eq. 3a/3b with a complex kernel (numpy.convolve), the real oracle when
every imaginary part is zero, the closed form of a pure rotation, an independently written
real 2x2-block recurrence, step == scan, chunk continuation, and finite differences of every
gradient (real and imaginary parts)."""
import numpy as np
import pytest

from oracle import complex_oracle as cx
from oracle import ss_oracle as orc


def _problem(seed, B=2, D=3, L=8, N=3):
    r = np.random.default_rng(seed)
    c = lambda *s: r.normal(size=s) + 1j * r.normal(size=s)
    return dict(u=r.normal(size=(B, D, L)), delta=r.normal(size=(B, D, L)) * 0.5, z=r.normal(size=(B, D, L)),
                A=-np.abs(r.normal(size=(D, N))) - 0.2 + 1j * r.normal(size=(D, N)) * 2.0,
                Bm=c(B, N, L), Cm=c(B, N, L), Dskip=r.normal(size=D), bias=r.normal(size=D) * 0.3, h0=c(B, D, N),
                dout=r.normal(size=(B, D, L)), dh_last=c(B, D, N))


def test_lti_case_is_a_convolution_with_a_complex_kernel():
    """Eq. 3a/3b: K_k = Re(sum_n C_n Abar_n^k Bbar_n), y = x * K, with S4D-Lin's A_n = -1/2 + n i."""
    r = np.random.default_rng(1)
    D, N, L = 2, 4, 20
    A = np.broadcast_to(-0.5 + 1j * np.arange(N), (D, N))
    Bc = r.normal(size=N) + 1j * r.normal(size=N)
    Cc = r.normal(size=N) + 1j * r.normal(size=N)
    step = np.array([0.07, 0.4])
    u = r.normal(size=(1, D, L))
    got = cx.scan_fwd(u, np.zeros_like(u), A, np.broadcast_to(Bc[None, :, None], (1, N, L)),
                      np.broadcast_to(Cc[None, :, None], (1, N, L)), bias=step)["out"]
    for d in range(D):
        abar = np.exp(step[d] * A[d])
        K = np.array([np.real(np.sum(Cc * abar ** k * step[d] * Bc)) for k in range(L)])
        np.testing.assert_allclose(got[0, d], np.convolve(u[0, d], K)[:L], rtol=1e-12, atol=1e-13)


def test_zero_imaginary_parts_give_the_real_oracle():
    p = _problem(2)
    real = {k: np.real(p[k]) for k in ("A", "Bm", "Cm", "h0", "dh_last")}
    kw = dict(Dskip=p["Dskip"], z=p["z"], bias=p["bias"], softplus=True)
    a = cx.scan_fwd(p["u"], p["delta"], real["A"], real["Bm"], real["Cm"], h0=real["h0"], **kw)
    b = orc.scan_fwd(p["u"], p["delta"], real["A"], real["Bm"], real["Cm"], h0=real["h0"], **kw)
    np.testing.assert_allclose(a["out"], b["out"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(a["h_last"], b["h_last"], rtol=1e-12, atol=1e-13)
    ga = cx.scan_bwd(p["u"], p["delta"], real["A"], real["Bm"], real["Cm"], p["dout"], h0=real["h0"],
                     dh_last=real["dh_last"], **kw)
    gb = orc.scan_bwd(p["u"], p["delta"], real["A"], real["Bm"], real["Cm"], p["dout"], h0=real["h0"],
                      dh_last=real["dh_last"], **kw)
    for k in ("du", "ddelta", "dz", "dD", "dbias"):
        np.testing.assert_allclose(ga[k], gb[k], rtol=1e-11, atol=1e-12)
    for k in ("dA", "dB", "dC", "dh0"):
        np.testing.assert_allclose(np.real(ga[k]), gb[k], rtol=1e-11, atol=1e-12)


def test_pure_rotation_closed_form():
    """A = i w, no input: h_t = exp(i w sum(dt)) h0, so |h| is preserved and y = Re(C h)."""
    L = 12
    w = 1.7
    dt = np.linspace(0.1, 0.4, L)[None, None, :]
    h0 = np.array([[[0.6 - 0.8j]]])
    ones = np.ones((1, 1, L), np.complex128)
    f = cx.scan_fwd(np.zeros((1, 1, L)), dt, np.array([[1j * w]]), ones, ones, h0=h0)
    want = np.real(np.exp(1j * w * np.cumsum(dt[0, 0])) * h0[0, 0, 0])
    np.testing.assert_allclose(f["out"][0, 0], want, rtol=1e-12, atol=1e-13)
    assert abs(abs(f["h_last"][0, 0, 0]) - 1.0) < 1e-12


def test_equals_a_real_two_by_two_block_recurrence():
    """(hr, hi) <- e^{dt ar} [[cos, -sin], [sin, cos]](dt ai) (hr, hi) + dt u (Br, Bi);  y = Cr hr - Ci hi."""
    p = _problem(3)
    f = cx.scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dskip=p["Dskip"], z=p["z"], bias=p["bias"],
                    h0=p["h0"], softplus=True)
    nb, nd, nl = p["u"].shape
    nn = p["A"].shape[1]
    for b in range(nb):
        for d in range(nd):
            hr, hi = np.real(p["h0"][b, d]).copy(), np.imag(p["h0"][b, d]).copy()
            for t in range(nl):
                r = p["delta"][b, d, t] + p["bias"][d]
                dt = np.log1p(np.exp(r))
                mag = np.exp(dt * np.real(p["A"][d]))
                c, s = np.cos(dt * np.imag(p["A"][d])), np.sin(dt * np.imag(p["A"][d]))
                hr, hi = (mag * (c * hr - s * hi) + dt * p["u"][b, d, t] * np.real(p["Bm"][b, :, t]),
                          mag * (s * hr + c * hi) + dt * p["u"][b, d, t] * np.imag(p["Bm"][b, :, t]))
                y = np.sum(np.real(p["Cm"][b, :, t]) * hr - np.imag(p["Cm"][b, :, t]) * hi) + p["Dskip"][d] * p["u"][b, d, t]
                zt = p["z"][b, d, t]
                assert f["out"][b, d, t] == pytest.approx(y * zt / (1 + np.exp(-zt)), rel=1e-12, abs=1e-13)
            np.testing.assert_allclose(f["h_last"][b, d], hr + 1j * hi, rtol=1e-12, atol=1e-13)


def test_step_and_chunks_equal_the_whole_scan():
    p = _problem(4, L=9)
    kw = dict(Dskip=p["Dskip"], bias=p["bias"], softplus=True)
    whole = cx.scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], z=p["z"], h0=p["h0"], **kw)
    h = p["h0"]
    for t in range(9):
        o, h = cx.step(h, p["u"][:, :, t], p["delta"][:, :, t], p["A"], p["Bm"][:, :, t], p["Cm"][:, :, t],
                       z_t=p["z"][:, :, t], **kw)
        np.testing.assert_allclose(o, whole["out"][:, :, t], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(h, whole["h_last"], rtol=1e-12, atol=1e-13)
    a = cx.scan_fwd(p["u"][:, :, :4], p["delta"][:, :, :4], p["A"], p["Bm"][:, :, :4], p["Cm"][:, :, :4],
                    z=p["z"][:, :, :4], h0=p["h0"], **kw)
    b = cx.scan_fwd(p["u"][:, :, 4:], p["delta"][:, :, 4:], p["A"], p["Bm"][:, :, 4:], p["Cm"][:, :, 4:],
                    z=p["z"][:, :, 4:], h0=a["h_last"], **kw)
    np.testing.assert_allclose(np.concatenate([a["out"], b["out"]], 2), whole["out"], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("softplus", [False, True])
def test_every_gradient_by_finite_differences(softplus):
    p = _problem(5)
    names = ["u", "delta", "z", "A", "Bm", "Cm", "Dskip", "bias", "h0"]
    gname = {"u": "du", "delta": "ddelta", "z": "dz", "A": "dA", "Bm": "dB", "Cm": "dC", "Dskip": "dD", "bias": "dbias",
             "h0": "dh0"}

    def loss(q):
        f = cx.scan_fwd(q["u"], q["delta"], q["A"], q["Bm"], q["Cm"], Dskip=q["Dskip"], z=q["z"], bias=q["bias"],
                        h0=q["h0"], softplus=softplus)
        return float(np.sum(f["out"] * p["dout"]) + np.sum(np.real(np.conj(p["dh_last"]) * f["h_last"])))
    g = cx.scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], p["dout"], Dskip=p["Dskip"], z=p["z"],
                    bias=p["bias"], h0=p["h0"], dh_last=p["dh_last"], softplus=softplus)
    r = np.random.default_rng(6)
    eps = 1e-6
    for name in names:
        arr = p[name]
        grad = g[gname[name]]
        assert grad.shape == arr.shape
        for _ in range(6):
            idx = tuple(r.integers(0, s) for s in arr.shape)
            for unit in ([1.0, 1j] if np.iscomplexobj(arr) else [1.0]):
                hi, lo = dict(p), dict(p)
                e = np.zeros(arr.shape, arr.dtype)
                e[idx] = unit * eps
                hi[name], lo[name] = arr + e, arr - e
                fd = (loss(hi) - loss(lo)) / (2 * eps)
                an = np.real(grad[idx]) if unit == 1.0 else np.imag(grad[idx])
                assert an == pytest.approx(fd, rel=2e-6, abs=1e-8), (name, idx, unit)
