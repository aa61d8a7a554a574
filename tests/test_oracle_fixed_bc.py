"""Pins of the oracle's time-invariant B / C modes (CPU only).

Algorithm 1 of the paper (S4) has B, C of shape (D,N) and a per-channel step size; the
ablation of Table 7 makes each of Delta, B, C selective or not.  The oracle takes a 2-D
(D,N) array for a time-invariant B or C.  Pins: the convolution form of Eq. 3a/3b with
numpy.convolve (fully time-invariant case), equality with the already pinned selective
path run channel by channel on broadcast copies (outputs and gradients, every mix of
fixed/selective), finite differences on the (D,N) parameters, and step == scan."""
import numpy as np
import pytest

from oracle import ss_oracle as orc


def _problem(seed, B=2, D=3, L=9, N=4):
    r = np.random.default_rng(seed)
    return dict(u=r.normal(size=(B, D, L)), delta=r.normal(size=(B, D, L)) * 0.5, z=r.normal(size=(B, D, L)),
                A=-np.abs(r.normal(size=(D, N))) - 0.2, Bsel=r.normal(size=(B, N, L)), Csel=r.normal(size=(B, N, L)),
                Bfix=r.normal(size=(D, N)), Cfix=r.normal(size=(D, N)), Dskip=r.normal(size=D),
                bias=r.normal(size=D) * 0.3, h0=r.normal(size=(B, D, N)), dout=r.normal(size=(B, D, L)),
                dh_last=r.normal(size=(B, D, N)))


@pytest.mark.parametrize("exact_zoh", [False, True])
def test_time_invariant_ssm_is_a_convolution(exact_zoh):
    """Eq. 3a/3b: K = (C Bbar, C Abar Bbar, ..., C Abar^k Bbar, ...), y = x * K."""
    p = _problem(1, B=2, D=3, L=17, N=4)
    step = np.array([0.05, 0.3, 1.1])                  # per-channel step size, as in Algorithm 1
    zeros = np.zeros_like(p["u"])
    got = orc.scan_fwd(p["u"], zeros, p["A"], p["Bfix"], p["Cfix"], bias=step, softplus=False,
                       exact_zoh=exact_zoh)["out"]
    for d in range(3):
        abar = np.exp(step[d] * p["A"][d])
        bbar = (abar - 1.0) / p["A"][d] * p["Bfix"][d] if exact_zoh else step[d] * p["Bfix"][d]
        K = np.array([np.sum(p["Cfix"][d] * abar ** k * bbar) for k in range(17)])
        for b in range(2):
            np.testing.assert_allclose(got[b, d], np.convolve(p["u"][b, d], K)[:17], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("bfix,cfix", [(True, True), (True, False), (False, True)])
@pytest.mark.parametrize("exact_zoh", [False, True])
def test_fixed_modes_equal_the_selective_path_channel_by_channel(bfix, cfix, exact_zoh):
    p = _problem(2)
    nb, nd, nl = p["u"].shape
    Bm = p["Bfix"] if bfix else p["Bsel"]
    Cm = p["Cfix"] if cfix else p["Csel"]
    kw = dict(softplus=True, exact_zoh=exact_zoh)
    f = orc.scan_fwd(p["u"], p["delta"], p["A"], Bm, Cm, Dskip=p["Dskip"], z=p["z"], bias=p["bias"], h0=p["h0"], **kw)
    g = orc.scan_bwd(p["u"], p["delta"], p["A"], Bm, Cm, p["dout"], Dskip=p["Dskip"], z=p["z"], bias=p["bias"],
                     h0=p["h0"], dh_last=p["dh_last"], **kw)
    assert g["dB"].shape == Bm.shape and g["dC"].shape == Cm.shape
    dB_sum = np.zeros_like(p["Bsel"])
    dC_sum = np.zeros_like(p["Csel"])
    for d in range(nd):
        sl = slice(d, d + 1)
        Bd = np.broadcast_to(p["Bfix"][d][None, :, None], p["Bsel"].shape) if bfix else p["Bsel"]
        Cd = np.broadcast_to(p["Cfix"][d][None, :, None], p["Csel"].shape) if cfix else p["Csel"]
        args = (p["u"][:, sl], p["delta"][:, sl], p["A"][sl], Bd, Cd)
        opt = dict(Dskip=p["Dskip"][sl], z=p["z"][:, sl], bias=p["bias"][sl], h0=p["h0"][:, sl])
        fd = orc.scan_fwd(*args, **opt, **kw)
        gd = orc.scan_bwd(*args, p["dout"][:, sl], dh_last=p["dh_last"][:, sl], **opt, **kw)
        np.testing.assert_allclose(f["out"][:, sl], fd["out"], rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(f["h_last"][:, sl], fd["h_last"], rtol=1e-13, atol=1e-14)
        for k in ("du", "ddelta", "dz", "dh0"):
            np.testing.assert_allclose(g[k][:, sl], gd[k], rtol=1e-12, atol=1e-13)
        for k in ("dA", "dD", "dbias"):
            np.testing.assert_allclose(g[k][sl], gd[k], rtol=1e-12, atol=1e-13)
        # a time-invariant parameter collects the gradient of all the positions it was broadcast to
        if bfix:
            np.testing.assert_allclose(g["dB"][d], gd["dB"].sum(axis=(0, 2)), rtol=1e-12, atol=1e-13)
        else:
            dB_sum += gd["dB"]
        if cfix:
            np.testing.assert_allclose(g["dC"][d], gd["dC"].sum(axis=(0, 2)), rtol=1e-12, atol=1e-13)
        else:
            dC_sum += gd["dC"]
    if not bfix:
        np.testing.assert_allclose(g["dB"], dB_sum, rtol=1e-12, atol=1e-13)
    if not cfix:
        np.testing.assert_allclose(g["dC"], dC_sum, rtol=1e-12, atol=1e-13)


def test_fixed_parameter_gradients_by_finite_differences():
    p = _problem(3)
    kw = dict(Dskip=p["Dskip"], z=p["z"], bias=p["bias"], h0=p["h0"], softplus=True)

    def loss(Bm, Cm):
        f = orc.scan_fwd(p["u"], p["delta"], p["A"], Bm, Cm, **kw)
        return float(np.sum(f["out"] * p["dout"]) + np.sum(f["h_last"] * p["dh_last"]))
    g = orc.scan_bwd(p["u"], p["delta"], p["A"], p["Bfix"], p["Cfix"], p["dout"], dh_last=p["dh_last"], **kw)
    eps = 1e-6
    for idx in np.ndindex(p["Bfix"].shape):
        e = np.zeros_like(p["Bfix"])
        e[idx] = eps
        fdB = (loss(p["Bfix"] + e, p["Cfix"]) - loss(p["Bfix"] - e, p["Cfix"])) / (2 * eps)
        fdC = (loss(p["Bfix"], p["Cfix"] + e) - loss(p["Bfix"], p["Cfix"] - e)) / (2 * eps)
        assert g["dB"][idx] == pytest.approx(fdB, rel=1e-6, abs=1e-8)
        assert g["dC"][idx] == pytest.approx(fdC, rel=1e-6, abs=1e-8)


@pytest.mark.parametrize("bfix,cfix", [(True, True), (True, False), (False, True)])
def test_fixed_modes_step_equals_scan(bfix, cfix):
    p = _problem(4, B=2, D=3, L=6, N=4)
    Bm = p["Bfix"] if bfix else p["Bsel"]
    Cm = p["Cfix"] if cfix else p["Csel"]
    whole = orc.scan_fwd(p["u"], p["delta"], p["A"], Bm, Cm, Dskip=p["Dskip"], z=p["z"], bias=p["bias"], h0=p["h0"],
                         softplus=True)
    h = p["h0"]
    for t in range(6):
        o, h = orc.step(h, p["u"][:, :, t], p["delta"][:, :, t], p["A"], Bm if bfix else Bm[:, :, t],
                        Cm if cfix else Cm[:, :, t], Dskip=p["Dskip"], z_t=p["z"][:, :, t], bias=p["bias"],
                        softplus=True, b_fixed=bfix, c_fixed=cfix)
        np.testing.assert_allclose(o, whole["out"][:, :, t], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(h, whole["h_last"], rtol=1e-12, atol=1e-13)
